"""Launch settings: per task (xs_app_desc.tuning) and process-wide; every setting leaves the
results bit-identical, only the launch shape changes."""
import numpy as np
import pytest
import torch

from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 12289, 50001, 2, 0, 70000]


def _task(dtype, W, align):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"ls_{dtype}", [(n,) for n in SIZES], W=W)
    t = harness.make_task(w, "cuda", align)
    t.momentum.copy_(wl.make_flat(t.n_bucket, 0.01, 5, device="cuda"))
    return w, t


def _settings(**kw):
    v = xs.tuning_preset(xs.PRESET_ALONE)
    for k, val in kw.items():
        v[getattr(xs, "TUNE_" + k)] = val
    return v


VARIANTS = {
    "beside": lambda: xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE),
    "leave wave slots": lambda: xs.tuning_preset(xs.PRESET_LEAVE_WAVE_SLOTS),
    "2 waves": lambda: _settings(REDUCE_WAVES_PER_WG=2, COPY_WAVES_PER_WG=2),
    "4 waves, persistent": lambda: _settings(REDUCE_WAVES_PER_WG=4, REDUCE_WG_PER_CU=2, COPY_WG_PER_CU=3,
                                             COPY_WAVES_PER_WG=4, COPY_LDS_RESERVE=40960, COPY_NT=0),
    "small kernel": lambda: _settings(REDUCE_SMALL=1),
    "4 waves, 7 workgroups": lambda: _settings(REDUCE_WAVES_PER_WG=4, REDUCE_MAX_WG=7, COPY_MAX_WG=5,
                                               COPY_WAVES_PER_WG=2),
}


@pytest.mark.parametrize("dtype,W", [("f32", 8), ("f16", 16), ("f32", 3), ("f16", 2)])
@pytest.mark.parametrize("form", ["packs", "gather", "fused_unpack"])
@pytest.mark.parametrize("variant", list(VARIANTS))
def test_per_task_settings_change_nothing_but_the_launch(dtype, W, form, variant):
    print(f"case settings dtype={dtype} W={W} form={form} variant={variant}", flush=True)
    w, ta = _task(dtype, W, 4)
    w, tb = _task(dtype, W, 4)
    kw = {"fused_gather": form == "gather", "fused_unpack": form == "fused_unpack"}
    a = ta.make_app(**kw)
    b = tb.make_app(tuning=VARIANTS[variant](), **kw)
    before = [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
    for _ in range(3):
        a.sync(); b.sync()
    torch.cuda.synchronize()
    assert [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)] == before     # per task, not global
    assert torch.equal(ta.params.view(torch.int32), tb.params.view(torch.int32))
    assert torch.equal(ta.momentum.view(torch.int32), tb.momentum.view(torch.int32))
    for p, q in zip(ta.param_tensors, tb.param_tensors):
        assert torch.equal(p, q)
    a.destroy(); b.destroy()


def test_invalid_settings_are_refused():
    w, t = _task("f32", 2, 4)
    bad = xs.tuning_preset(xs.PRESET_ALONE)
    bad[xs.TUNE_REDUCE_WAVES_PER_WG] = 3
    with pytest.raises(xs.XsError) as e:
        t.make_app(tuning=bad)
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    with pytest.raises(xs.XsError):
        xs.tuning_set(xs.TUNE_REDUCE_WAVES_PER_WG, 3)
    with pytest.raises(xs.XsError):
        xs.tuning_preset(7)
    pre = xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE)
    assert pre[xs.TUNE_REDUCE_WAVES_PER_WG] == 4 and pre[xs.TUNE_REDUCE_SMALL] == 1 and pre[xs.TUNE_COPY_WAVES_PER_WG] == 4
    assert xs.tuning_preset(xs.PRESET_ALONE) == [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
