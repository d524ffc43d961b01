"""Host-side checks of the C-ABI library that need no GPU: the library loads, exports
every function the header declares, and rejects bad arguments before launching."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2103_07974_amd import xs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "xs.h")

FAKE = 0x7f0000001000          # never dereferenced: validation fails first


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xs_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    L = xs.lib()
    names = _declared_functions()
    assert {"xs_fuse_pack", "xs_fused_reduce_sgd", "xs_fuse_unpack", "xs_crossover_step"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(xs.EXPORTS)


def test_status_strings():
    assert xs.status_string(0) == "XS_OK"
    assert xs.status_string(-2) == "XS_ERR_ALIGNMENT"
    assert xs.status_string(-99) == "XS_ERR_UNKNOWN"


@pytest.mark.parametrize("align", [1, 2, 4, 64, 100])
def test_layout_matches_oracle(align):
    rng = np.random.default_rng(align)
    numel = [int(v) for v in rng.integers(0, 5000, size=40)] + [0, 1, 64, 4096]
    assert xs.bucket_layout(numel, align) == [int(v) for v in oracle.layout(numel, align)]


def test_layout_errors():
    with pytest.raises(xs.XsError) as e:
        xs.bucket_layout([1, 2], 0)
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    assert xs.bucket_layout([], 8) == [0]


def _reduce(W=2, dtype=xs.XS_F32, n=16, params=FAKE, mom=FAKE + 0x1000, pout=None, mout=None,
            reps=None, hp=True, flag=None):
    L = xs.lib()
    reps = [FAKE + 0x10000 * (i + 2) for i in range(W)] if reps is None else reps
    arr = (ctypes.c_void_p * max(len(reps), 1))(*reps)
    h = xs.SgdHparams(0.1, 0.9, 0.0, 1.0)
    return L.xs_fused_reduce_sgd(arr, W, dtype, n, params, mom, pout, mout,
                                 ctypes.byref(h) if hp else None, flag, None)


def test_reduce_argument_validation():
    assert _reduce(W=0) == xs.XS_ERR_INVALID_ARG
    assert _reduce(W=xs.XS_MAX_REPLICAS + 1) == xs.XS_ERR_INVALID_ARG
    assert "W = 33" in xs.last_error()
    assert _reduce(dtype=7) == xs.XS_ERR_UNSUPPORTED
    assert _reduce(hp=False) == xs.XS_ERR_INVALID_ARG
    assert _reduce(params=None) == xs.XS_ERR_INVALID_ARG
    assert _reduce(params=FAKE + 4) == xs.XS_ERR_ALIGNMENT
    assert _reduce(mom=FAKE + 0x1008) == xs.XS_ERR_ALIGNMENT
    assert _reduce(reps=[FAKE + 0x20000, FAKE + 0x30002]) == xs.XS_ERR_ALIGNMENT
    assert _reduce(reps=[FAKE + 0x20000, None]) == xs.XS_ERR_INVALID_ARG
    assert _reduce(pout=FAKE + 0x4000, mout=None) == xs.XS_ERR_INVALID_ARG
    assert _reduce(flag=FAKE + 0x9002) == xs.XS_ERR_ALIGNMENT
    # aliasing: momentum inside params, a replica on top of params
    assert _reduce(mom=FAKE + 16, n=16) == xs.XS_ERR_INVALID_ARG
    assert _reduce(reps=[FAKE, FAKE + 0x20000]) == xs.XS_ERR_INVALID_ARG
    assert _reduce(pout=FAKE + 0x1000, mout=FAKE + 0x5000) == xs.XS_ERR_INVALID_ARG
    # n_elems == 0 is a valid no-op even with no buffers
    assert _reduce(n=0, params=None, mom=None) == xs.XS_OK


def test_pack_unpack_reject_bad_handles():
    L = xs.lib()
    assert L.xs_fuse_pack(None, FAKE, FAKE, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_fuse_unpack(None, FAKE, FAKE, None) == xs.XS_ERR_INVALID_ARG
    junk = ctypes.create_string_buffer(256)
    assert L.xs_fuse_pack(ctypes.addressof(junk), FAKE, FAKE, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_plan_destroy(None) == xs.XS_OK
    assert L.xs_app_destroy(None) == xs.XS_OK
    assert L.xs_plan_bucket_elems(None) == 0
    assert L.xs_crossover_step(None, None, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_crossover_drain(None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_app_sync(None, None) == xs.XS_ERR_INVALID_ARG


def test_plan_create_validates_before_touching_the_device():
    L = xs.lib()
    h = ctypes.c_void_p()
    u64 = ctypes.c_uint64

    def create(numel, offsets, dtype=xs.XS_F32):
        a = (u64 * max(len(numel), 1))(*numel)
        o = (u64 * len(offsets))(*offsets)
        return L.xs_plan_create(a, o, len(numel), dtype, ctypes.byref(h))

    assert create([4, 4], [0, 4, 6]) == xs.XS_ERR_SIZE          # second tensor overruns
    assert "overruns" in xs.last_error()
    assert create([4, 4], [0, 8, 4]) == xs.XS_ERR_SIZE          # not monotone
    assert create([4], [1, 5]) == xs.XS_ERR_SIZE                # must start at 0
    assert create([4], [0, 4], dtype=9) == xs.XS_ERR_UNSUPPORTED
    assert L.xs_plan_create(None, None, 0, 0, ctypes.byref(h)) == xs.XS_ERR_INVALID_ARG
    assert L.xs_plan_create(None, None, 0, 0, None) == xs.XS_ERR_INVALID_ARG


def test_tuning_roundtrip_and_range():
    old = xs.tuning_get(xs.TUNE_REDUCE_WG_PER_CU)
    xs.tuning_set(xs.TUNE_REDUCE_WG_PER_CU, 4)
    assert xs.tuning_get(xs.TUNE_REDUCE_WG_PER_CU) == 4
    xs.tuning_set(xs.TUNE_REDUCE_WG_PER_CU, old)
    with pytest.raises(xs.XsError):
        xs.tuning_set(xs.TUNE_REDUCE_WG_PER_CU, 1000)
    with pytest.raises(xs.XsError):
        xs.tuning_set(99, 1)
    assert xs.tuning_get(xs.TUNE_REDUCE_LDS_RESERVE) == -1      # per-dtype default
    with pytest.raises(xs.XsError):
        xs.tuning_set(xs.TUNE_NT_GRADS, 2)
    with pytest.raises(xs.XsError):
        xs.tuning_set(xs.N_TUNING_KEYS, 0)


def test_header_tuning_enum_matches_binding():
    text = open(HEADER).read()
    for name, value in re.findall(r"XS_(TUNE_[A-Z_]+) = (\d+)", text):
        if name == "TUNE_COUNT":
            assert int(value) == xs.N_TUNING_KEYS
        else:
            assert getattr(xs, name) == int(value), name


def test_mixed_precision_option_validation():
    L = xs.lib()
    arr = (ctypes.c_void_p * 2)(FAKE + 0x20000, FAKE + 0x30000)
    h = xs.SgdHparams(0.1, 0.9, 0.0, 1.0)

    def reduce_mp(copy, dt):
        mp = xs.MpOptions(copy, dt, 0)
        return L.xs_fused_reduce_sgd_mp(arr, 2, xs.XS_F32, 16, FAKE, FAKE + 0x1000, None, None,
                                        ctypes.byref(h), None, ctypes.byref(mp), None)
    assert reduce_mp(FAKE + 0x5000, xs.XS_F32) == xs.XS_ERR_UNSUPPORTED      # not a half type
    assert reduce_mp(FAKE + 0x5002, xs.XS_F16) == xs.XS_ERR_ALIGNMENT
    assert reduce_mp(FAKE + 0x1000, xs.XS_BF16) == xs.XS_ERR_INVALID_ARG     # on top of momentum
    assert reduce_mp(FAKE + 0x20010, xs.XS_F16) == xs.XS_ERR_INVALID_ARG     # on top of a replica
    # the live half-precision model must not be written by a pass that may still be skipped:
    # out-of-place outputs + found_inf (in-kernel detection) + model_copy is refused
    mp = xs.MpOptions(FAKE + 0x5000, xs.XS_F16, 0)
    rc = L.xs_fused_reduce_sgd_mp(arr, 2, xs.XS_F16, 16, FAKE, FAKE + 0x1000, FAKE + 0x2000, FAKE + 0x3000,
                                  ctypes.byref(h), FAKE + 0x7000, ctypes.byref(mp), None)
    assert rc == xs.XS_ERR_UNSUPPORTED and "model_copy" in xs.last_error()


def test_pool_layout():
    sizes = [1, 2 << 20, (2 << 20) + 1, 0, 553430272]
    offs = xs.pool_layout(sizes)
    assert offs[0] == 0 and len(offs) == len(sizes) + 1
    for i, n in enumerate(sizes):
        assert offs[i] % xs.POOL_ALIGN == 0 and offs[i + 1] >= offs[i] + n and offs[i + 1] - offs[i] < n + xs.POOL_ALIGN + 1
    assert offs[-1] == sum((n + xs.POOL_ALIGN - 1) // xs.POOL_ALIGN * xs.POOL_ALIGN for n in sizes)
    assert xs.pool_layout([]) == [0]
    L = xs.lib()
    assert L.xs_pool_layout(None, 0, None) == xs.XS_ERR_INVALID_ARG
    big = (ctypes.c_uint64 * 2)(2 ** 63, 2 ** 63); out = (ctypes.c_uint64 * 3)()
    assert L.xs_pool_layout(big, 2, out) == xs.XS_ERR_SIZE


def test_launch_settings_presets_and_atomics():
    L = xs.lib()
    alone, beside = xs.tuning_preset(xs.PRESET_ALONE), xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE)
    assert len(alone) == xs.N_TUNING_KEYS and alone == [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
    assert beside[xs.TUNE_REDUCE_WAVES_PER_WG] == 4 and beside[xs.TUNE_REDUCE_LDS_RESERVE] == 82 * 1024
    assert L.xs_tuning_preset(0, None) == xs.XS_ERR_INVALID_ARG
    slots = xs.tuning_preset(xs.PRESET_LEAVE_WAVE_SLOTS)
    assert [k for k in range(xs.N_TUNING_KEYS) if slots[k] != alone[k]] == [xs.TUNE_COPY_LDS_RESERVE]
    assert slots[xs.TUNE_COPY_LDS_RESERVE] == 16 * 1024
    with pytest.raises(xs.XsError):
        xs.tuning_preset(3)
    for bad in (0, 3, 5):
        with pytest.raises(xs.XsError):
            xs.tuning_set(xs.TUNE_REDUCE_WAVES_PER_WG, bad)
    # plan-less pack: layout errors and the size limit are found before anything touches a device
    n = xs.STATIC_MAX_TENSORS + 1
    numel = (ctypes.c_uint64 * n)(*([1] * n)); offs = (ctypes.c_uint64 * (n + 1))(*range(n + 1))
    assert L.xs_fuse_pack_static(numel, offs, n, xs.XS_F32, FAKE, FAKE + 0x1000, None, None) == xs.XS_ERR_SIZE
    assert "XS_STATIC_MAX_TENSORS" in xs.last_error()
    assert L.xs_fuse_pack_static(numel, offs, 2, 7, FAKE, FAKE + 0x1000, None, None) == xs.XS_ERR_UNSUPPORTED
    assert L.xs_fuse_pack_static(None, None, 2, xs.XS_F32, FAKE, FAKE + 0x1000, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_fuse_pack_static(numel, offs, 0, xs.XS_F32, None, None, None, None) == xs.XS_OK


def test_per_tensor_and_n_task_entry_points_reject_bad_handles():
    L = xs.lib()
    arr = (ctypes.c_void_p * 2)(FAKE + 0x20000, FAKE + 0x30000)
    junk = ctypes.create_string_buffer(256)
    for plan in (None, ctypes.addressof(junk)):
        assert L.xs_fused_reduce_sgd_pt(plan, arr, 2, FAKE, FAKE + 0x1000, None, None, FAKE + 0x8000,
                                        1.0, None, None, None) == xs.XS_ERR_INVALID_ARG
        assert L.xs_fused_gather_reduce_sgd_pt(plan, FAKE, 2, FAKE, FAKE + 0x1000, None, None, None,
                                               FAKE + 0x8000, 1.0, None, None, None) == xs.XS_ERR_INVALID_ARG
    assert "plan" in xs.last_error()
    # N-task loop: an empty array is a no-op, anything else must be apps
    assert L.xs_crossover_iteration(None, 0, None, None) == xs.XS_OK
    assert L.xs_crossover_finish(None, 0, None) == xs.XS_OK
    assert L.xs_crossover_iteration(None, 2, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_crossover_finish(None, 2, None) == xs.XS_ERR_INVALID_ARG
    apps = (ctypes.c_void_p * 2)(ctypes.addressof(junk), None)
    assert L.xs_crossover_iteration(apps, 2, None, None) == xs.XS_ERR_INVALID_ARG
    assert L.xs_crossover_finish(apps, 2, None) == xs.XS_ERR_INVALID_ARG
    assert "apps[0]" in xs.last_error()


def test_header_record_is_sixteen_bytes_of_floats():
    # the binding builds the per-tensor table as rows of four float32
    text = open(HEADER).read()
    start = text.index("typedef struct {\n    float lr;\n    float momentum;\n    float weight_decay;\n    float reserved;")
    assert "} xs_tensor_hparams;" in text[start:start + 300]


def test_header_is_valid_c99_and_usable_from_c(tmp_path):
    """The boundary is a C interface: the header must compile as strict C99 and a C program
    must be able to call the library through it (host-only entry points here)."""
    import subprocess
    src = tmp_path / "use_xs.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "xs.h"
int main(void)
{
    uint64_t numel[3] = {5, 0, 130}, offs[4];
    xs_sgd_hparams hp = {0.1f, 0.9f, 1e-4f, 1.0f};
    xs_tensor_hparams rec = {0.1f, 0.9f, 0.0f, 0.0f};
    xs_mp_options mp = {0, XS_F16, XS_F32};
    xs_app_desc desc;
    memset(&desc, 0, sizeof desc);
    (void)hp; (void)rec; (void)mp;
    if (sizeof(rec) != 16) return 2;
    if (xs_bucket_layout(numel, 3, 64, offs) != XS_OK) return 3;
    if (offs[1] != 64 || offs[2] != 64 || offs[3] != 256) return 4;
    if (xs_bucket_layout(numel, 3, 0, offs) != XS_ERR_INVALID_ARG) return 5;
    if (strstr(xs_last_error(), "align_elems") == NULL) return 6;
    if (xs_fuse_pack(NULL, NULL, NULL, NULL, NULL) != XS_ERR_INVALID_ARG) return 7;
    if (xs_crossover_iteration(NULL, 0, NULL, NULL) != XS_OK) return 8;
    printf("%s\n", xs_status_string(XS_ERR_STATE));
    return 0;
}
''')
    exe = tmp_path / "use_xs"
    libdir = os.path.dirname(xs.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.dirname(HEADER),
           str(src), "-o", str(exe), "-L", libdir, "-lxs", f"-Wl,-rpath,{libdir}",
           "-Wl,-rpath,/opt/rocm/lib", "-L", "/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    assert res.stdout.strip() == "XS_ERR_STATE"
