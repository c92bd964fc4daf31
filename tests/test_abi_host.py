"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/eco.h declares, validates its arguments before touching the device, and derives the
step constants as documented."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def eco():
    lib_path = os.path.join(ROOT, "paper_2601_22101_amd", "libeco.so")
    if not os.path.exists(lib_path):
        from paper_2601_22101_amd import build
        build.build()
    from paper_2601_22101_amd import binding
    return binding


def test_every_declared_symbol_is_exported(eco):
    header = open(os.path.join(ROOT, "include", "eco.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(eco_[a-z_0-9]+)\s*\(", header))
    assert {"eco_plan_create", "eco_plan_destroy", "eco_step", "eco_step_tensors", "eco_step_tensors_noalloc", "eco_quantize_init",
            "eco_dequantize", "eco_quantize_error", "eco_bandwidth_probe", "eco_arith_selftest", "eco_philox_fill", "eco_step_constants", "eco_set_option", "eco_status_string",
            "eco_last_error", "eco_version"} <= names
    for n in names:
        assert hasattr(eco.lib, n), n
    assert eco.eco_version() >= 100
    assert eco.eco_status_string(0) == "ok" and "align" in eco.eco_status_string(eco.ECO_EALIGN)


def test_struct_layouts_match_header(eco):
    assert C.sizeof(eco.eco_tensor_t) == 72
    assert C.sizeof(eco.eco_hparams_t) == 80
    assert C.sizeof(eco.eco_constants_t) == 52


def _tensor(eco, **kw):
    base = dict(weights=0x1000, scales=0x2000, grad=0x3000, m=0x4000, v=0x5000, numel=4096, tensor_id=0,
                fmt=eco.ECO_FMT_FP8_E4M3, aux=None, group_size=0)
    base.update(kw)
    return eco.make_tensor(**base)


def _status(eco, fn, *args):
    try:
        fn(*args)
    except eco.EcoError as e:
        return e.status
    return 0


def test_plan_validation_happens_before_any_device_work(eco):
    hp = eco.make_hparams()
    bad = [
        (dict(numel=0), eco.ECO_EINVAL),
        (dict(weights=None), eco.ECO_EINVAL),
        (dict(grad=None), eco.ECO_EINVAL),
        (dict(m=None), eco.ECO_EINVAL),
        (dict(v=None), eco.ECO_EINVAL),              # Adam needs v
        (dict(scales=None), eco.ECO_EINVAL),         # quantized format needs scales
        (dict(fmt=7), eco.ECO_EINVAL),
        (dict(weights=0x1008), eco.ECO_EALIGN),
        (dict(m=0x4004), eco.ECO_EALIGN),
        (dict(grad=0x3002), eco.ECO_EALIGN),
    ]
    for kw, want in bad:
        assert _status(eco, eco.eco_plan_create, [_tensor(eco, **kw)], hp) == want, kw
        assert eco.eco_last_error()
    assert _status(eco, eco.eco_plan_create, [], hp) == eco.ECO_EINVAL
    for bs, want in ((0, eco.ECO_EINVAL), (16, eco.ECO_EUNSUPPORTED), (100, eco.ECO_EUNSUPPORTED),
                     (1024, eco.ECO_EUNSUPPORTED)):
        assert _status(eco, eco.eco_plan_create, [_tensor(eco)], eco.make_hparams(block_size=bs)) == want
    assert _status(eco, eco.eco_plan_create, [_tensor(eco)], eco.make_hparams(state_dtype=5)) == eco.ECO_EINVAL
    # per-tensor scale groups: powers of two in [32, 512], multiples of 8 up to 8192, or the whole tensor
    for gs in (100, 12, 1004):
        assert _status(eco, eco.eco_plan_create, [_tensor(eco, group_size=gs)], hp) == eco.ECO_EUNSUPPORTED, gs
    assert _status(eco, eco.eco_plan_create, [_tensor(eco, numel=20000, group_size=9000)], hp) == eco.ECO_EUNSUPPORTED
    # the master-weight and exact-injection modes need the aux buffer, aligned
    for mode, opt in ((eco.ECO_MODE_MASTER, eco.ECO_OPT_ADAM), (eco.ECO_MODE_EXACT, eco.ECO_OPT_SGDM)):
        hp2 = eco.make_hparams(mode=mode, opt=opt)
        assert _status(eco, eco.eco_plan_create, [_tensor(eco)], hp2) == eco.ECO_EINVAL
        assert _status(eco, eco.eco_plan_create, [_tensor(eco, aux=0x6004)], hp2) == eco.ECO_EALIGN
    assert _status(eco, eco.eco_plan_create, [_tensor(eco, aux=0x6000)],
                   eco.make_hparams(mode=eco.ECO_MODE_EXACT)) == eco.ECO_EUNSUPPORTED
    # SGDM does not need v
    st = _status(eco, eco.eco_plan_create, [_tensor(eco, v=None)], eco.make_hparams(opt=eco.ECO_OPT_SGDM))
    assert st in (eco.ECO_OK, eco.ECO_EHIP, eco.ECO_ENOMEM)      # passes validation; no GPU here -> HIP error


def test_noalloc_step_refuses_what_its_static_scratch_cannot_hold(eco):
    """Limits of the allocation-free plan-less step are checked on the host, before any device work."""
    hp = eco.make_hparams()
    t = _tensor(eco)
    assert _status(eco, eco.eco_step_tensors_noalloc, [t] * 4097, hp, 0) == eco.ECO_EUNSUPPORTED
    assert "4096" in eco.eco_last_error()
    assert _status(eco, eco.eco_step_tensors_noalloc, [_tensor(eco, numel=(1 << 29) + 512)], hp, 0) == eco.ECO_EUNSUPPORTED
    assert _status(eco, eco.eco_step_tensors_noalloc, [_tensor(eco, numel=1 << 28)] * 3, hp, 0) == eco.ECO_EUNSUPPORTED
    # one scale group per table entry for groups wider than 512 elements
    assert _status(eco, eco.eco_step_tensors_noalloc, [_tensor(eco, numel=(1 << 20) * 520 + 520, group_size=520)], hp, 0) == eco.ECO_EUNSUPPORTED
    # and the usual validation comes first
    assert _status(eco, eco.eco_step_tensors_noalloc, [_tensor(eco, m=None)], hp, 0) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_step_tensors_noalloc, [_tensor(eco, grad=0x3004)], hp, 0) == eco.ECO_EALIGN
    assert _status(eco, eco.eco_step_tensors_noalloc, [t], eco.make_hparams(step=0), 0) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_step_tensors_noalloc, [t], eco.make_hparams(block_size=100), 0) == eco.ECO_EUNSUPPORTED
    assert _status(eco, eco.eco_step_tensors_noalloc, [], hp, 0) == eco.ECO_EINVAL


def test_hparams_validation(eco):
    ok = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1)
    eco.eco_step_constants(eco.make_hparams(**ok))
    for kw in (dict(step=0), dict(lr=0.0), dict(lr=-1.0), dict(lr=float("nan")), dict(beta1=0.0), dict(beta1=1.0),
               dict(beta2=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(weight_decay=-0.1), dict(opt=3),
               dict(round=2), dict(mode=4), dict(mode=-1), dict(state_dtype=9)):
        assert _status(eco, eco.eco_step_constants, eco.make_hparams(**{**ok, **kw})) == eco.ECO_EINVAL, kw
    # without injection nothing divides by lr or beta1
    eco.eco_step_constants(eco.make_hparams(**{**ok, "lr": 0.0, "inject": False}))
    eco.eco_step_constants(eco.make_hparams(**{**ok, "beta1": 0.0, "inject": False}))
    # the validation precedes the plan in the plan-less entry point as well
    assert _status(eco, eco.eco_step_tensors, [_tensor(eco)], eco.make_hparams(step=0), 0) == eco.ECO_EINVAL


def test_flat_helpers_validate(eco):
    q = lambda **kw: _status(eco, eco.eco_quantize_init, kw.get("src", 0x1000), kw.get("sdt", 0), kw.get("n", 1024),
                             kw.get("fmt", 0), kw.get("bs", 128), kw.get("scdt", 0), kw.get("w", 0x2000),
                             kw.get("s", 0x3000), 0)
    assert q(n=0) == eco.ECO_EINVAL
    assert q(src=None) == eco.ECO_EINVAL
    assert q(w=None) == eco.ECO_EINVAL
    assert q(fmt=2) == eco.ECO_EINVAL
    assert q(bs=100) == eco.ECO_EUNSUPPORTED
    assert q(bs=0) == eco.ECO_EINVAL
    assert q(src=0x1004) == eco.ECO_EALIGN
    assert q(n=(1 << 40) + 1) == eco.ECO_EUNSUPPORTED          # size guard, before any launch
    assert q(n=1 << 35) == eco.ECO_EUNSUPPORTED                # one launch holds fewer than 2^32 threads: 2^26 tiles are one too many
    assert q(n=1 << 35, bs=1 << 36) == eco.ECO_EUNSUPPORTED    # the same for one scale over the tensor
    assert q(n=1 << 35, bs=520) == eco.ECO_EUNSUPPORTED        # wide groups: a workgroup of two waves for every 520 elements
    assert _status(eco, eco.eco_dequantize, 0x1000, 0x2000, 1 << 35, 0, 128, 0, 0x3000, 0) == eco.ECO_EUNSUPPORTED
    assert _status(eco, eco.eco_bandwidth_probe, 0, 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 1 << 35, 0) == eco.ECO_EINVAL
    assert q(bs=8200, n=1 << 20) == eco.ECO_EUNSUPPORTED       # wide groups end at 8192 elements ...
    assert q(bs=20, n=1 << 20) == eco.ECO_EUNSUPPORTED         # ... and are multiples of 8
    assert _status(eco, eco.eco_dequantize, 0x1000, 0x2000, 1024, 0, 128, 0, None, 0) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_dequantize, 0x1000, 0x2000, 100, 0, 7, 0, 0x3000, 0) == eco.ECO_EUNSUPPORTED
    qe = lambda **kw: _status(eco, eco.eco_quantize_error, *[{**dict(src=0x1000, sd=0, w=0x2000, s=0x3000, n=1024, fmt=0, gs=128,
                                                                     sc=0, err=0x4000, st=0), **kw}[k]
                                                            for k in ("src", "sd", "w", "s", "n", "fmt", "gs", "sc", "err", "st")])
    assert qe(src=None) == eco.ECO_EINVAL and qe(err=None) == eco.ECO_EINVAL and qe(w=None) == eco.ECO_EINVAL
    assert qe(err=0x4004) == eco.ECO_EALIGN and qe(src=0x1008) == eco.ECO_EALIGN
    assert qe(fmt=2) == eco.ECO_EINVAL and qe(sd=9) == eco.ECO_EINVAL and qe(n=0) == eco.ECO_EINVAL
    assert qe(gs=4) == eco.ECO_EUNSUPPORTED
    assert _status(eco, eco.eco_philox_fill, 1, 1, 0, 0, 0, 0x1000, 0) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_philox_fill, 1, 1, 0, 0, 16, None, 0) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_set_option, 5, 1) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_set_option, 0, 100000) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_set_option, 2, 40000) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_set_option, 3, 100) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_set_option, 3, 2 ** 32) == eco.ECO_EINVAL
    eco.eco_set_option(3, 4096)
    eco.eco_set_option(3, -1)
    eco.eco_set_option(0, 0)
    eco.eco_set_option(2, -1)


def test_step_constants_follow_the_paper(eco):
    """kappa = ((1-b1^k)/lr)(1-1/b1) (Alg. 3 line 5), alpha = (1/lr)(1-1/b) (Eq. alpha), the Adam step
    lr/(1-b1^k) and 1/(1-b2^k) (Sec. 3.2): formed in double, rounded once to fp32."""
    for lr, b1, b2, eps, wd, k in ((1e-3, 0.9, 0.999, 1e-8, 0.0, 1), (3e-4, 0.9, 0.98, 1e-9, 0.1, 17),
                                   (1e-5, 0.95, 0.999, 1e-8, 0.01, 100000)):
        c = eco.eco_step_constants(eco.make_hparams(lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=wd, step=k))
        f = np.float32
        bc1, bc2 = 1 - b1 ** k, 1 - b2 ** k
        assert c.b1 == f(b1) and c.omb1 == f(1 - b1) and c.b2 == f(b2) and c.omb2 == f(1 - b2)
        assert c.eps == f(eps) and c.lr == f(lr) and c.wd == f(lr * wd)
        for got, want in ((c.rbc2, 1 / bc2), (c.c1, lr / bc1), (c.kappa, (bc1 / lr) * (1 - 1 / b1)),
                          (c.alpha, (1 / lr) * (1 - 1 / b1))):
            assert abs(got - want) <= abs(want) * 2.0 ** -23
        assert c.kappa < 0 and c.alpha < 0
    c = eco.eco_step_constants(eco.make_hparams(inject=False))
    assert c.kappa == 0 and c.alpha == 0 and c.inv_lr == 0
    # exact stored-error injection (Appendix A): 1/eta and 1/(eta beta); SGDM only
    c = eco.eco_step_constants(eco.make_hparams(opt=eco.ECO_OPT_SGDM, mode=eco.ECO_MODE_EXACT, lr=0.05, beta1=0.9))
    assert c.kappa == 0 and c.alpha == 0
    assert abs(c.inv_lr - 20.0) < 1e-5 and abs(c.inv_lr_beta - 1 / 0.045) < 1e-5
    assert _status(eco, eco.eco_step_constants, eco.make_hparams(mode=eco.ECO_MODE_EXACT)) == eco.ECO_EUNSUPPORTED
    c = eco.eco_step_constants(eco.make_hparams(mode=eco.ECO_MODE_MASTER))
    assert c.kappa == 0 and c.alpha == 0 and c.inv_lr == 0
    # doubles that are valid one by one but leave the fp32 range once combined are refused: the injection strength
    # (1/lr)(1 - 1/beta) of a tiny learning rate, the Adam step lr/(1-b1^k) of a huge one
    assert _status(eco, eco.eco_step_constants, eco.make_hparams(lr=1e-42)) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_step_constants, eco.make_hparams(opt=eco.ECO_OPT_SGDM, lr=1e-40, beta1=0.5)) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_step_constants, eco.make_hparams(lr=1e39, inject=False)) == eco.ECO_EINVAL
    assert _status(eco, eco.eco_step_constants, eco.make_hparams(lr=1e-30, inject=False)) == 0      # no division by lr without injection


def test_product_package_never_reaches_the_oracle():
    """The product path must not import, read or link anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2601_22101_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for fn in files:
            if fn.endswith((".py", ".cpp", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), fn
                assert "eco_oracle" not in text and "liboracle" not in text, fn


def test_harness_arena_layout_is_aligned_and_fits_its_pool(eco):
    """Host logic of the harness: every tensor's slice of every arena starts 256-byte aligned, slices do not
    overlap, and one allocation of pool_bytes holds all arenas (with any number of gradient sets)."""
    import workloads
    from paper_2601_22101_amd.harness import DeviceWorkload as D
    for wl in (workloads.config2(), workloads.config4(), workloads.config5(),
               workloads.with_granularity(workloads.config4(), "row"),
               workloads.with_granularity(workloads.config5(), "tensor")):
        offs, soffs, coffs, woffs, off, soff, code_bytes, woff = D._layout(wl)
        st = 2 if wl.state_bf16 else 4
        sc = 2 if wl.scale_bf16 else 4
        prev_end = {"e": 0, "s": 0, "c": 0, "w": 0}
        for t, o, so, co, wo in zip(wl.tensors, offs, soffs, coffs, woffs):
            assert o % 512 == 0 and o >= prev_end["e"]
            prev_end["e"] = o + t.numel
            if t.fmt in ("fp8", "int4"):
                gs = t.group_size(wl.block_size)
                assert (so * sc) % 256 == 0 and so >= prev_end["s"]
                prev_end["s"] = so + (t.numel + gs - 1) // gs
                assert co % 256 == 0 and co >= prev_end["c"]
                prev_end["c"] = co + (t.numel if t.fmt == "fp8" else (t.numel + 1) // 2)
            else:
                assert wo % 512 == 0 and wo >= prev_end["w"]
                prev_end["w"] = wo + t.numel
        assert prev_end["e"] <= off and prev_end["s"] <= max(soff, 1) and prev_end["c"] <= max(code_bytes, 1)
        for mode, sets in ((eco.ECO_MODE_ECO, 1), (eco.ECO_MODE_MASTER, 1), (eco.ECO_MODE_ECO, 8)):
            arenas = [max(code_bytes, 1), max(soff, 1) * sc, max(woff, 1) * 2, st * off, st * off] + [2 * off] * sets
            if mode == eco.ECO_MODE_MASTER:
                arenas.append(4 * off)
            # each arena starts on a 2 MiB boundary inside the pool
            need = sum(-(-a // (1 << 21)) * (1 << 21) for a in arenas) + (1 << 21)
            assert D.pool_bytes(wl, mode, sets) >= need


def test_harness_candidate_orders_use_every_arena_once():
    """Host logic of the probed placement: every candidate order is a permutation of the same arenas (so none leaves a
    byte unused or an arena out), units stay together and in their order, the candidates are distinct, and between
    them v follows m at every possible distance."""
    from paper_2601_22101_amd.harness import DeviceWorkload as D
    for fillers in ([["codes", "scales", "plain"], ["grad"]],
                    [["codes", "scales", "plain"]] + [[f"g{k}"] for k in range(8)],
                    [["codes", "scales", "plain"], ["grad"], ["grad_extra1"], ["aux"]]):
        names = sorted(["m", "v"] + [n for u in fillers for n in u])
        orders = D.candidate_orders(fillers)
        F = len(fillers)
        assert len(orders) == 2 * F - 1 and len({tuple(o) for o in orders}) == len(orders)
        gaps = set()
        for o in orders:
            assert sorted(o) == names
            assert o.index("m") < o.index("v")
            rest = [n for n in o if n not in ("m", "v")]
            assert rest == [n for u in fillers for n in u]                 # the other arenas keep their order
            for u in fillers:                                              # and a unit is never split by m or v
                i = o.index(u[0])
                assert o[i:i + len(u)] == u
            assert o[0] == "m" or o[-1] == "v"
            gaps.add((o[0] == "m", sum(1 for u in fillers if o.index("m") < o.index(u[0]) < o.index("v"))))
        assert {g for first, g in gaps if first} == set(range(1, F + 1))
        assert {g for first, g in gaps if not first} == set(range(1, F))


def test_launch_geometry_host_checks(tmp_path):
    """The geometry the library derives from a tensor's scale group (kernel class, rows to a workgroup, what one
    helper launch holds), compiled for the host alone and checked over every group length: tests/native/geometry_host.cpp."""
    import subprocess
    exe = str(tmp_path / "geometry_host")
    cmd = ["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I", os.path.join(ROOT, "paper_2601_22101_amd", "csrc"), os.path.join(ROOT, "tests", "native", "geometry_host.cpp"), "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert out.returncode == 0 and "geometry ok" in out.stdout, out.stdout


def test_a_plain_c_client_compiles_links_and_runs(eco, tmp_path):
    """include/eco.h is valid C99 (-Wall -Wextra -pedantic -Werror), libeco.so links by its C names, and the
    host-only entry points give a C caller what they give the Python binding."""
    import subprocess
    lib_dir = os.path.join(ROOT, "paper_2601_22101_amd")
    exe = str(tmp_path / "abi_host")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "native", "abi_host.c"), "-o", exe, "-L", lib_dir, "-l:libeco.so",
           f"-Wl,-rpath,{lib_dir}"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert out.returncode == 0, out.stdout
    lines = dict(l.split(" ", 1) for l in out.stdout.strip().splitlines())
    assert lines["version"] == str(eco.eco_version())
    assert lines["sizes"] == "72 80 52"
    vals = lines["constants"].split()
    assert vals[0] == "0"
    hp = eco.make_hparams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=3, seed=7, block_size=128)
    c = eco.eco_step_constants(hp)
    ref = [c.b1, c.omb1, c.b2, c.omb2, c.rbc2, c.c1, c.eps, c.kappa]
    assert [np.float32(float(x)) for x in vals[1:]] == [np.float32(x) for x in ref]
    assert lines["step0"].startswith(f"{eco.ECO_EINVAL} invalid argument |") and "1-based" in lines["step0"]
    assert lines["nullplan"] == str(eco.ECO_EINVAL) and lines["destroynull"] == "0"
