"""eco_step_tensors_noalloc, the plan-less step for callers that cannot allocate device memory, against
eco_step_tensors through the C ABI: same inputs, same hyper-parameters, on two calls in a row of which the second
is smaller (the static scratch then still holds the first call's tables beyond what the second one rewrites).

The bar is the one of every parity test here (tests/gpu_util.py): codes and scales bit-exact, m and v within 1e-6
relative; both entry points run the same kernels, so the check asks for identical bytes.
"""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def mixed_workload(n_small):
    """Block-scaled FP8 and INT4 tensors with ragged tails, row-wise groups that fill and do not fill their
    workgroup, tensors with a single scale (one tile, many tiles, a ragged end), bf16 norm vectors: every launch
    list of the step, and more than 32 tensors so that the table kernel runs more than once."""
    T = workloads.TensorSpec
    ts = [T("a", (192, 1024)), T("b", (2048 * 3 + 77,)), T("c", (7,)), T("i4", (300, 256), "int4"), T("i4r", (4099,), "int4"),
          T("norm", (512,), "bf16_plain"), T("norm_r", (1000,), "bf16_plain"),
          T("row1024", (96, 1024), granularity="row"), T("row1408", (40, 1408), granularity="row"),
          T("row24", (50, 24), granularity="row"), T("i4row", (64, 2048), "int4", granularity="row"),
          T("tw_small", (4096,), granularity="tensor"), T("tw_big", (700, 1000), granularity="tensor"),
          T("tw_ragged", (300001,), granularity="tensor"), T("i4tw", (200, 1024), "int4", granularity="tensor")]
    ts += [T(f"s{i}", (1024 + 512 * (i % 5) + 8 * i,), "fp8" if i % 3 else "int4", grad_std=1e-3 * (1 + i % 4))
           for i in range(n_small)]
    return workloads.Workload("noalloc_mixed", ts, steps=2)


def snapshot(dw):
    torch.cuda.synchronize()
    return [(tv.weights.clone(), None if tv.scales is None else tv.scales.clone(), tv.m.clone(), tv.v.clone())
            for tv in dw.tensors]


def assert_same(a, b, wl, what):
    for tv, ta, tb in zip(wl.tensors, a, b):
        for name, x, y in zip(("weights", "scales", "m", "v"), ta, tb):
            if x is None:
                continue
            assert torch.equal(x, y), f"{what}: {tv.name} {name} differs"
            if name in ("m", "v"):
                assert bool(torch.isfinite(x).all())


def test_noalloc_step_equals_the_allocating_one_twice_in_a_row():
    from paper_2601_22101_amd import binding as eco
    from paper_2601_22101_amd import harness
    big, small = mixed_workload(40), mixed_workload(0)
    small.tensors = small.tensors[1:9:2] + small.tensors[11:13]        # fewer and other tensors, other list offsets
    for wl, steps in ((big, (1, 2)), (small, (3,))):                   # three calls in a row: large, large, smaller
        ref = harness.DeviceWorkload(wl, DEV)
        dut = harness.DeviceWorkload(wl, DEV)
        assert_same(snapshot(ref), snapshot(dut), wl, "set-up")
        for k in steps:
            ref.fill_gradients(k)
            dut.fill_gradients(k)
            hp = ref.hparams(k)
            eco.eco_step_tensors([ref.descriptor(tv) for tv in ref.tensors], hp)
            before = snapshot(dut)
            eco.eco_step_tensors_noalloc([dut.descriptor(tv) for tv in dut.tensors], hp)
            after = snapshot(dut)
            assert_same(snapshot(ref), after, wl, f"{wl.name} ({len(wl.tensors)} tensors) step {k}")
            changed = sum(not torch.equal(x[2], y[2]) for x, y in zip(before, after))
            assert changed == len(wl.tensors), "every tensor of the call must have been stepped"
        ref.close()
        dut.close()


def test_noalloc_step_other_variants_and_limits():
    """SGDM with nearest rounding and bf16 state on the same scratch right after an Adam call; sizes beyond the
    static scratch are refused before anything is launched."""
    from paper_2601_22101_amd import binding as eco
    from paper_2601_22101_amd import harness
    wl = mixed_workload(3)
    wl.state_bf16 = wl.scale_bf16 = True
    over = dict(opt=eco.ECO_OPT_SGDM, round=eco.ECO_ROUND_RTN, lr=0.05)
    ref = harness.DeviceWorkload(wl, DEV, layout=over)
    dut = harness.DeviceWorkload(wl, DEV, layout=over)
    for k in (1, 2):
        ref.fill_gradients(k)
        dut.fill_gradients(k)
        hp = ref.hparams(k)
        eco.eco_step_tensors([ref.descriptor(tv) for tv in ref.tensors], hp)
        eco.eco_step_tensors_noalloc([dut.descriptor(tv) for tv in dut.tensors], hp)
        assert_same(snapshot(ref), snapshot(dut), wl, f"sgdm/rtn/bf16 step {k}")
    d = dut.descriptor(dut.tensors[0])
    hp = dut.hparams(3)
    before = snapshot(dut)
    with pytest.raises(eco.EcoError) as e:
        eco.eco_step_tensors_noalloc([d] * 4097, hp)
    assert e.value.status == eco.ECO_EUNSUPPORTED and "4096" in str(e.value)
    huge = eco.make_tensor(d.weights, d.scales, d.grad, d.m, d.v, (1 << 29) + 512, 0, 0)    # 2^20 + 1 tiles: never touched
    with pytest.raises(eco.EcoError) as e:
        eco.eco_step_tensors_noalloc([huge], hp)
    assert e.value.status == eco.ECO_EUNSUPPORTED
    assert_same(before, snapshot(dut), wl, "a refused call must not have run anything")
    ref.close()
    dut.close()
