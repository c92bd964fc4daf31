"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by element
on the same seeded inputs.  Sizes span several 2048-element tiles and ragged tails; the bar is in
tests/gpu_util.py."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from oracle import FMT_E4M3, FMT_INT4

from gpu_util import bf16_bits, compare, host_copy, oracle_step, step_config, to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eco():
    from paper_2601_22101_amd import binding
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


@pytest.fixture(scope="module")
def harness():
    from paper_2601_22101_amd import harness
    return harness


DEV = "cuda:0"


# ---------------------------------------------------------------------------------- building blocks

def test_philox_stream_is_bit_exact(eco, o32):
    for seed, step, tid, first, n in ((0, 1, 0, 0, 4096), (0x0123456789ABCDEF, 7, 42, 0, 1000),
                                      (99, 3, 5, 13, 3001), (5, 2 ** 32 + 9, 1, (1 << 34) - 6, 64)):
        dst = torch.zeros(n, dtype=torch.int32, device=DEV)
        eco.eco_philox_fill(seed, step, tid, first, n, dst)
        got = dst.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, o32.philox_fill(seed, step, tid, n, first_word=first)), (seed, step, tid, first)


@pytest.mark.parametrize("fmt", [0, 1])
def test_the_step_uses_every_bit_of_seed_step_and_tensor_id(eco, o32, fmt):
    """The largest values the counter words take: seed 2^64 - 1 and other 64-bit seeds, tensor_id 2^32 - 1, steps beyond
    2^31 and 2^32 (only the low word enters the counter; the bias corrections have long since reached 1).  The step's own
    random stream must be the oracle's for all of them."""
    from types import SimpleNamespace
    n = 3 * 512 + 200
    gen = torch.Generator(device=DEV)
    gen.manual_seed(3)
    src = torch.randn(n, device=DEV, generator=gen) * 0.02
    for seed, step, tid in ((2 ** 64 - 1, 1, 2 ** 32 - 1), (0x8000000000000001, 2 ** 31 + 5, 0x80000000),
                            (0xFEDCBA9876543210, 2 ** 32 + 3, 0xFFFF0000), (0, 2 ** 40 + 1, 1)):
        codes = torch.zeros(n if fmt == 0 else n // 2, dtype=torch.uint8, device=DEV)
        scales = torch.zeros((n + 127) // 128, dtype=torch.float32, device=DEV)
        eco.eco_quantize_init(src, eco.ECO_DT_FP32, n, fmt, 128, eco.ECO_DT_FP32, codes, scales)
        grad = (torch.randn(n, device=DEV, generator=gen) * 1e-3).to(torch.bfloat16)
        m = torch.randn(n, device=DEV, generator=gen) * 1e-3
        v = torch.rand(n, device=DEV, generator=gen) * 1e-6
        tv = SimpleNamespace(weights=codes, scales=scales, grad=grad, m=m, v=v, aux=None)
        h = host_copy(tv)
        hp = eco.make_hparams(lr=1e-3, step=step, seed=seed)
        eco.eco_step_tensors([eco.make_tensor(codes, scales, grad, m, v, n, tid, fmt)], hp)
        torch.cuda.synchronize()
        oracle_step(o32, h, n, step_config(hp, tid, fmt))
        st = compare(host_copy(tv), h, f"seed {seed:#x} step {step} tensor_id {tid:#x}")
        assert st["code_mismatch"] == 0 and st["m_bit_mismatch"] == 0, st


def test_short_square_root_and_division_are_correctly_rounded(eco):
    """The step kernels use shorter sequences than sqrtf() and `/` inside stated operand ranges; the library's self-test
    compares short and long form on the device: every fp32 argument of the square root's range (1.6e9 patterns), and
    every denominator of the division's range (8.1e8 patterns) for several numerators c1 = lr / (1 - beta1^k), typical
    and extreme -- 6.5e9 operand pairs, every exponent difference the short form can meet."""
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    eco.eco_arith_selftest(0, 0.0, 0x0F800000, 0x6F800001, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0, "short square root differs from sqrtf"
    for c1 in (1e-3, 1e-3 / (1 - 0.9), 1e-5 / (1 - 0.9 ** 3), 3e-4 / (1 - 0.9 ** 7), 2.0 ** -40, 2.0 ** 40, 0.7853982, -1.9999999):
        eco.eco_arith_selftest(1, c1, 0x27800000, 0x58000001, bad)
        torch.cuda.synchronize()
        assert int(bad.item()) == 0, f"short division differs from / for numerator {c1}"
    # the entry point refuses operands outside the ranges the short forms are used in
    for args in ((0, 0.0, 0x0F7FFFFF, 0x10000000), (1, 1.0, 0x27800000, 0x58000002), (1, 2.0 ** 41, 0x30000000, 0x30000010),
                 (2, 1.0, 0x30000000, 0x30000010), (1, 1.0, 0x30000010, 0x30000010)):
        with pytest.raises(eco.EcoError):
            eco.eco_arith_selftest(*args, bad)


def test_bandwidth_probe_touches_what_it_says_and_nothing_else(eco):
    """The measurement aid moves real bytes: the plain copy copies m to v; the byte-mix copy swaps m and v, mixes the
    gradient into the codes, rewrites the scales with their own values and leaves the gradient alone; neither writes
    a byte beyond the `numel` elements it was given (guard regions before and after every array)."""
    n, guard = 8 * 1024, 1024
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)

    def arr(count, dtype):
        if dtype.is_floating_point:         # finite values: the probe passes m through one floating-point addition of zero
            full = torch.randn(count + 2 * guard, dtype=dtype, device=DEV, generator=gen) + 3.0
        else:
            full = torch.randint(0, 255, ((count + 2 * guard) * torch.empty(0, dtype=dtype).element_size(),), dtype=torch.uint8,
                                 device=DEV, generator=gen).view(dtype)
        return full, full[guard:guard + count]
    codes_f, codes = arr(n, torch.uint8)
    scales_f, scales = arr(n // 128, torch.float32)
    grad_f, grad = arr(n, torch.int16)
    m_f, m = arr(n, torch.float32)
    v_f, v = arr(n, torch.float32)
    m_f, v_f, m, v = m_f.view(torch.int32), v_f.view(torch.int32), m.view(torch.int32), v.view(torch.int32)
    before = {k: t.clone() for k, t in dict(codes=codes_f, scales=scales_f.view(torch.int32), grad=grad_f, m=m_f, v=v_f).items()}
    eco.eco_bandwidth_probe(1, None, None, None, m, v, n)
    torch.cuda.synchronize()
    assert torch.equal(v, m) and torch.equal(m_f, before["m"])
    assert torch.equal(v_f[:guard], before["v"][:guard]) and torch.equal(v_f[guard + n:], before["v"][guard + n:])
    assert torch.equal(codes_f, before["codes"]) and torch.equal(grad_f, before["grad"])
    v_f.copy_(before["v"])
    eco.eco_bandwidth_probe(0, codes, scales, grad, m, v, n)
    torch.cuda.synchronize()
    b = {k: t[guard:guard + c] for (k, t), c in zip(before.items(), (n, n // 128, n, n, n))}
    assert torch.equal(m, b["v"]) and torch.equal(v, b["m"]), "m and v swap"
    assert torch.equal(scales.view(torch.int32), b["scales"]) and torch.equal(grad, b["grad"])
    g = b["grad"].view(torch.int32).view(-1, 4)                     # a lane's 8 gradients: four dwords
    want = b["codes"].view(torch.int32).view(-1, 2) ^ torch.stack([g[:, 0] ^ g[:, 2], g[:, 1] ^ g[:, 3]], dim=1)
    assert torch.equal(codes.view(torch.int32).view(-1, 2), want)
    for name, full, count in (("codes", codes_f, n), ("scales", scales_f.view(torch.int32), n // 128), ("grad", grad_f, n),
                              ("m", m_f, n), ("v", v_f, n)):
        assert torch.equal(full[:guard], before[name][:guard]) and torch.equal(full[guard + count:], before[name][guard + count:]), name


@pytest.mark.parametrize("fmt", [0, 1])
@pytest.mark.parametrize("bf16", [False, True])
def test_no_entry_point_writes_outside_its_arrays(eco, fmt, bf16):
    """Every array of every tensor sits between two guard regions of random bytes, with no padding after its last element:
    the initial quantizer, the step (block-scaled tensors with ragged tails, rows that do not fill their workgroup, a
    ragged last row, one scale per tensor; through a plan, plan-less and allocation-free), the de-quantizer and the
    error call must leave every guard byte as it was -- and the read-only gradient too."""
    guard = 4096
    gen = torch.Generator(device=DEV)
    gen.manual_seed(17 + fmt + 2 * bf16)
    sdt = torch.bfloat16 if bf16 else torch.float32
    dt = eco.ECO_DT_BF16 if bf16 else eco.ECO_DT_FP32
    held = []

    def arr(nbytes):
        """nbytes of payload between two guards; returns the payload as a uint8 view (16-byte aligned start)."""
        full = torch.randint(0, 256, (guard + nbytes + guard,), dtype=torch.uint8, device=DEV, generator=gen)
        held.append((full, full.clone(), nbytes))
        return full[guard:guard + nbytes]

    cases = [(1, 128), (7, 128), (127, 32), (513, 128), (4097, 64), (12345, 512), (5 * 1000, 1000), (3 * 520, 520),
             (2 * 1000 + 40, 1000), (2 * 8192 + 8, 8192), (100, 1 << 20), (70001, 1 << 20), (8193, 8193)]
    tensors, payload = [], []
    for tid, (numel, gs) in enumerate(cases):
        if fmt == 1 and numel % 2:
            numel += 1                                   # INT4 packs two codes a byte; an odd tail shares its byte
            if gs >= numel - 1:
                gs = max(gs, numel)                      # ... and one scale for the tensor stays one scale
        ngroups = (numel + gs - 1) // gs
        codes = arr(numel if fmt == 0 else numel // 2)
        scales = arr(ngroups * (2 if bf16 else 4)).view(sdt)
        grad = arr(2 * numel).view(torch.bfloat16)
        m = arr(numel * (2 if bf16 else 4)).view(sdt)
        v = arr(numel * (2 if bf16 else 4)).view(sdt)
        src = arr(4 * numel).view(torch.float32)
        out = arr(4 * numel).view(torch.float32)
        src.copy_(torch.randn(numel, device=DEV, generator=gen) * 0.02)
        grad.copy_((torch.randn(numel, device=DEV, generator=gen) * 1e-3).to(torch.bfloat16))
        m.copy_((torch.randn(numel, device=DEV, generator=gen) * 1e-3).to(sdt))
        v.copy_((torch.rand(numel, device=DEV, generator=gen) * 1e-6).to(sdt))
        eco.eco_quantize_init(src, eco.ECO_DT_FP32, numel, fmt, gs, dt, codes, scales)
        tensors.append(eco.make_tensor(codes, scales, grad, m, v, numel, tid, fmt, group_size=gs))
        payload.append((numel, gs, codes, scales, grad, m, v, src, out))
    torch.cuda.synchronize()
    for full, ref, nbytes in held:                       # set-up is done: from here on the guards must not move
        ref.copy_(full)
    grads = [p[4].clone() for p in payload]
    hp = lambda k: eco.make_hparams(block_size=128, state_dtype=dt, scale_dtype=dt, lr=1e-3, step=k, seed=9)
    with eco.Plan(tensors, hp(1)) as plan:
        plan.step(hp(1))
    eco.eco_step_tensors(tensors, hp(2))
    eco.eco_step_tensors_noalloc(tensors, hp(3))
    for numel, gs, codes, scales, grad, m, v, src, out in payload:
        eco.eco_dequantize(codes, scales, numel, fmt, gs, dt, out)
        eco.eco_quantize_error(src, eco.ECO_DT_FP32, codes, scales, numel, fmt, gs, dt, out)
    torch.cuda.synchronize()
    for full, ref, nbytes in held:
        assert torch.equal(full[:guard], ref[:guard]), "bytes before an array were written"
        assert torch.equal(full[guard + nbytes:], ref[guard + nbytes:]), "bytes after an array were written"
    for (numel, gs, codes, scales, grad, m, v, src, out), g0 in zip(payload, grads):
        assert torch.equal(grad.view(torch.int16), g0.view(torch.int16)), "the gradient is read-only"
        assert bool(torch.isfinite(m.float()).all()) and bool(torch.isfinite(out).all())


def test_decode_every_code(eco, o32):
    codes = torch.arange(256, dtype=torch.uint8, device=DEV)
    scales = torch.ones(2, dtype=torch.float32, device=DEV)
    out = torch.zeros(256, dtype=torch.float32, device=DEV)
    eco.eco_dequantize(codes, scales, 256, eco.ECO_FMT_FP8_E4M3, 128, eco.ECO_DT_FP32, out)
    got, ref = out.cpu().numpy(), o32.decode_table(FMT_E4M3)
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok].view(np.uint32), ref[ok].view(np.uint32))
    nib = torch.tensor([0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE] * 4, dtype=torch.uint8, device=DEV)
    out = torch.zeros(64, dtype=torch.float32, device=DEV)
    eco.eco_dequantize(nib, scales, 64, eco.ECO_FMT_INT4, 32, eco.ECO_DT_FP32, out)
    assert np.array_equal(out.cpu().numpy()[:16], o32.decode_table(FMT_INT4))


@pytest.mark.parametrize("fmt", [0, 1])
@pytest.mark.parametrize("scale_bf16", [False, True])
@pytest.mark.parametrize("numel,bs", [(1024 * 1024, 128), (2048 * 3 + 1000, 128), (4099, 32), (5000, 64),
                                      (777, 256), (9000, 512), (7, 128)])
def test_quantize_init_matches_oracle(eco, o32, fmt, scale_bf16, numel, bs):
    g = torch.Generator().manual_seed(numel + bs)
    x = torch.randn(numel, generator=g) * 0.02
    x[::97] = 0.0
    if numel > 3000:
        x[2048:2048 + bs] = 0.0                       # an all-zero block
        x[1024:1024 + bs] *= 1e-30                    # a block whose scale underflows towards zero
    sdt = torch.bfloat16 if scale_bf16 else torch.float32
    nb = (numel + bs - 1) // bs
    xd = x.to(DEV)
    codes = torch.zeros(numel if fmt == 0 else (numel + 1) // 2, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(nb, dtype=sdt, device=DEV)
    eco.eco_quantize_init(xd, eco.ECO_DT_FP32, numel, fmt, bs, int(scale_bf16), codes, scales)
    rc, rs = o32.quantize_rtn(fmt, x.numpy(), block_size=bs, scale_bf16=scale_bf16)
    assert np.array_equal(codes.cpu().numpy(), rc)
    assert np.array_equal(to_f32(scales).view(np.uint32), rs.view(np.uint32))
    # and back
    out = torch.zeros(numel, dtype=torch.float32, device=DEV)
    eco.eco_dequantize(codes, scales, numel, fmt, bs, int(scale_bf16), out)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), o32.dequantize(fmt, rc, rs, numel, bs).view(np.uint32))
    # bf16 source
    xb = x.to(torch.bfloat16)
    eco.eco_quantize_init(xb.to(DEV), eco.ECO_DT_BF16, numel, fmt, bs, int(scale_bf16), codes, scales)
    rc, rs = o32.quantize_rtn(fmt, xb.float().numpy(), block_size=bs, scale_bf16=scale_bf16)
    assert np.array_equal(codes.cpu().numpy(), rc)


@pytest.mark.parametrize("seed", range(64))
def test_randomized_quantize_and_dequantize(eco, o32, seed):
    """Seeded random (length, scale group, source and scale type): the initial quantizer and the dequantizer
    against the oracle, for every class of group (in-wave block, wide group, whole tensor, ragged ends)."""
    rng = np.random.default_rng(5000 + seed)
    fmt = int(rng.integers(0, 2))
    numel = int(rng.choice([1, 5, 8, 100, 511, 512, 8192, 8193, 12345, int(rng.integers(1, 200000))]))
    kind = rng.choice(["block", "wide", "tensor"])
    if kind == "block":
        gs = int(rng.choice([32, 64, 128, 256, 512]))
    elif kind == "wide":
        gs = 8 * int(rng.integers(1, 1025))
    else:
        gs = numel + int(rng.integers(0, 3)) * 1000
    if fmt == 1 and gs % 2 and gs < numel:
        gs += 1
    scale_bf16, src_bf16 = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    x = torch.from_numpy((rng.standard_normal(numel) * 10.0 ** rng.uniform(-6, 2)).astype(np.float32))
    x[rng.integers(0, numel, size=max(1, numel // 50))] = 0.0
    if src_bf16:
        x = x.to(torch.bfloat16)
    ng = (numel + min(gs, numel) - 1) // min(gs, numel)
    codes = torch.zeros(numel if fmt == 0 else (numel + 1) // 2, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(ng, dtype=torch.bfloat16 if scale_bf16 else torch.float32, device=DEV)
    eco.eco_quantize_init(x.to(DEV), int(src_bf16), numel, fmt, gs, int(scale_bf16), codes, scales)
    rc, rs = o32.quantize_rtn(fmt, x.float().numpy(), block_size=min(gs, numel), scale_bf16=scale_bf16)
    what = (seed, fmt, numel, gs, scale_bf16, src_bf16)
    assert np.array_equal(codes.cpu().numpy(), rc), what
    assert np.array_equal(to_f32(scales).view(np.uint32), rs.view(np.uint32)), what
    out = torch.zeros(numel, dtype=torch.float32, device=DEV)
    eco.eco_dequantize(codes, scales, numel, fmt, gs, int(scale_bf16), out)
    ref = o32.dequantize(fmt, rc, rs, numel, min(gs, numel))
    assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), what
    # the quantization error e = theta - q(theta) (Sec. 3.1 notation; the e_0 of Appendix A): one fp32 subtraction
    err = torch.full((numel,), 7.0, dtype=torch.float32, device=DEV)
    eco.eco_quantize_error(x.to(DEV), int(src_bf16), codes, scales, numel, fmt, gs, int(scale_bf16), err)
    want = x.float().numpy() - ref
    assert want.dtype == np.float32 and np.array_equal(err.cpu().numpy().view(np.uint32), want.view(np.uint32)), what


def test_tensorwise_quantize_calls_may_overlap_on_two_streams(eco, o32):
    """One scale per tensor needs the tensor's abs-max between two kernels of a call; calls on different streams
    must not see each other's.  Many calls, alternating between two streams and more of them than the library
    has slots, against the oracle."""
    rng = np.random.default_rng(77)
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    jobs = []
    for k in range(150):
        numel = int(rng.integers(9000, 400000))
        fmt = int(rng.integers(0, 2))
        x = torch.from_numpy((rng.standard_normal(numel) * 10.0 ** rng.uniform(-4, 1)).astype(np.float32))
        jobs.append((numel, fmt, x, x.to(DEV), torch.zeros(numel if fmt == 0 else (numel + 1) // 2, dtype=torch.uint8, device=DEV),
                     torch.zeros(1, dtype=torch.float32, device=DEV)))
    torch.cuda.synchronize()
    for k, (numel, fmt, x, xd, codes, scale) in enumerate(jobs):
        eco.eco_quantize_init(xd, eco.ECO_DT_FP32, numel, fmt, numel, eco.ECO_DT_FP32, codes, scale, stream=streams[k & 1])
    torch.cuda.synchronize()
    for k, (numel, fmt, x, xd, codes, scale) in enumerate(jobs):
        rc, rs = o32.quantize_rtn(fmt, x.numpy(), block_size=numel)
        assert np.array_equal(codes.cpu().numpy(), rc), k
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), rs.view(np.uint32)), k


# ---------------------------------------------------------------------------------- whole workloads

def run_workload_parity(harness, o32, wl, steps, base_seed=workloads.BASE_SEED, **over):
    """Every tensor, every step: the library on the device, the oracle on host copies of the same bits."""
    dw = harness.DeviceWorkload(wl, DEV, base_seed)
    host = [host_copy(tv) for tv in dw.tensors]
    # the initial round-to-nearest quantization is itself part of the path: check it against the oracle's
    for tv, h in zip(dw.tensors, host):
        if tv.scales is not None:
            w0 = workloads.initial_weights(wl, tv.tensor_id, device=DEV, base_seed=base_seed).cpu().numpy()
            rc, rs = o32.quantize_rtn(oracle.FMT_E4M3 if tv.fmt == 0 else oracle.FMT_INT4, w0, dw.group_size(tv),
                                      wl.scale_bf16)
            assert np.array_equal(h["codes"], rc) and np.array_equal(h["scales"].view(np.uint32), rs.view(np.uint32))
    worst = {}
    for k in range(1, steps + 1):
        dw.fill_gradients(k)
        hp = dw.hparams(k, **over)
        for tv, h in zip(dw.tensors, host):
            h["grad"] = bf16_bits(tv.grad)
        dw.plan.step(hp)
        torch.cuda.synchronize()
        for tv, h in zip(dw.tensors, host):
            oracle_step(o32, h, tv.spec.numel, step_config(hp, tv.tensor_id, tv.fmt, group_size=dw.group_size(tv)))
            st = compare(host_copy(tv), h, f"{wl.name} step {k} tensor {tv.spec.name}", wl.state_bf16)
            for key, val in st.items():
                worst[key] = max(worst.get(key, 0), val)
    dw.close()
    return worst


def test_config1_every_step(harness, o32):
    worst = run_workload_parity(harness, o32, workloads.config1(), steps=10)
    assert worst["code_mismatch"] == 0 and worst["m_bit_mismatch"] == 0 and worst["v_bit_mismatch"] == 0, worst


def test_config2_multi_tensor_every_step(harness, o32):
    wl = workloads.config2()
    worst = run_workload_parity(harness, o32, wl, steps=wl.steps)
    assert worst["code_mismatch"] == 0, worst


def small_mixed_workload(fmt="fp8", **kw):
    """A few tensors of awkward sizes: below one tile, ragged tiles, ragged blocks, odd lengths."""
    T = workloads.TensorSpec
    sizes = [(64, 1024), (3, 2048), (2048 * 2 + 128 * 5,), (128 * 9 + 40,), (7,), (4097,), (1,), (2048,), (513, 9)]
    ts = [T(f"t{i}", s, fmt, grad_std=1e-3 * (1 + i)) for i, s in enumerate(sizes)]
    ts.insert(3, T("norm", (512,), "bf16_plain"))
    ts.insert(6, T("norm_ragged", (1000,), "bf16_plain"))
    return workloads.Workload("mixed_" + fmt, ts, steps=4, **kw)


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
@pytest.mark.parametrize("opt,rnd,inject,wd", [(0, 0, True, 0.0), (0, 1, True, 0.0), (1, 0, True, 0.0),
                                               (1, 1, True, 0.1), (0, 0, False, 0.0), (0, 0, True, 0.1)])
def test_variants_on_ragged_tensors(harness, o32, fmt, opt, rnd, inject, wd):
    wl = small_mixed_workload(fmt)
    over = dict(opt=opt, round=rnd, inject=inject, weight_decay=wd)
    if opt == 1:
        over["lr"] = 0.05
    # the plan is built from hparams(1) of the workload, which is Adam: rebuild for SGDM
    dw_over = dict(over)
    worst = _run_with_layout(harness, o32, wl, 4, dw_over)
    assert worst["code_mismatch"] == 0, worst


def _run_with_layout(harness, o32, wl, steps, over):
    dw = harness.DeviceWorkload(wl, DEV, layout=over)
    over = {}
    host = [host_copy(tv) for tv in dw.tensors]
    worst = {}
    for k in range(1, steps + 1):
        dw.fill_gradients(k)
        hp = dw.hparams(k, **over)
        for tv, h in zip(dw.tensors, host):
            h["grad"] = bf16_bits(tv.grad)
        dw.plan.step(hp)
        torch.cuda.synchronize()
        for tv, h in zip(dw.tensors, host):
            oracle_step(o32, h, tv.spec.numel, step_config(hp, tv.tensor_id, tv.fmt, group_size=dw.group_size(tv)))
            st = compare(host_copy(tv), h, f"{wl.name} step {k} {tv.spec.name} {over}", wl.state_bf16)
            for key, val in st.items():
                worst[key] = max(worst.get(key, 0), val)
    dw.close()
    return worst


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
@pytest.mark.parametrize("grad_std,over", [(1e-17, {}), (1e-20, {}), (1e18, {}), (1e-3, dict(lr=1e-14)), (1e-3, dict(lr=1e-3, eps=2.0)),
                                           (1e-3, dict(lr=50.0, beta1=0.5)), (1e-3, dict(eps=0.0, beta2=0.0))])
def test_operands_outside_the_short_forms_take_the_long_ones(harness, o32, fmt, grad_std, over):
    """The kernels use short square-root and division sequences inside operand ranges and sqrtf / `/` outside them; here
    the operands are outside: second moments below 2^-96 (gradients of 1e-17), denormal ones (1e-20), above 2^96 (1e18), a
    numerator eta / (1 - beta1^k) below 2^-40, epsilon above 1, a huge learning rate, and beta2 = epsilon = 0.  Every code,
    scale and state value must still be the oracle's."""
    T = workloads.TensorSpec
    ts = [T("a", (8, 1024), fmt, grad_std=grad_std), T("ragged", (4097,), fmt, grad_std=grad_std),
          T("rows", (6, 1000), fmt, grad_std=grad_std, granularity="row"), T("whole", (20000,), fmt, grad_std=grad_std, granularity="tensor"),
          T("mixed", (4096,), fmt, grad_std=1e-3), T("norm", (600,), "bf16_plain", grad_std=grad_std)]
    wl = workloads.Workload("extremes_" + fmt, ts, steps=3)
    worst = _run_with_layout(harness, o32, wl, 3, dict(over))
    assert worst["code_mismatch"] == 0 and worst["m_bit_mismatch"] == 0 and worst["v_bit_mismatch"] == 0, worst


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
@pytest.mark.parametrize("opt,mode,rnd", [(0, 3, 0), (0, 3, 1), (1, 3, 0), (1, 2, 0), (1, 2, 1)])
def test_master_weight_and_exact_injection_modes(harness, o32, fmt, opt, mode, rnd):
    """ECO_MODE_MASTER (fp32 master copy, Sec. 3.1) and ECO_MODE_EXACT (stored error, Appendix A) on ragged tensors."""
    wl = small_mixed_workload(fmt)
    over = dict(opt=opt, mode=mode, round=rnd)
    if opt == 1:
        over["lr"] = 0.05
    worst = _run_with_layout(harness, o32, wl, 4, over)
    assert worst["code_mismatch"] == 0 and worst["aux_bit_mismatch"] == 0, worst


def test_exact_injection_tracks_master_weights_on_the_device(harness, eco):
    """Appendix A on the GPU: from the theorem's initial conditions the stored-error run and the master-weight
    run see the same gradients and must keep (almost always) the same codes; theta^ + e tracks the master copy."""
    wl = workloads.Workload("eq", [workloads.TensorSpec("w", (64, 1024))], steps=8, lr=0.05)
    a = harness.DeviceWorkload(wl, DEV, layout=dict(opt=eco.ECO_OPT_SGDM, mode=eco.ECO_MODE_MASTER, round=eco.ECO_ROUND_RTN))
    b = harness.DeviceWorkload(wl, DEV, layout=dict(opt=eco.ECO_OPT_SGDM, mode=eco.ECO_MODE_EXACT, round=eco.ECO_ROUND_RTN))
    n = wl.numel
    deq = torch.zeros(n, device=DEV)
    b.tensors[0].m.copy_(-b.tensors[0].aux / (0.05 * wl.beta1))      # m_0 = m_0^MW - e_0/(eta beta), m_0^MW = 0
    for k in range(1, 9):
        a.fill_gradients(k)
        b.fill_gradients(k)
        a.step(k)
        b.step(k)
        torch.cuda.synchronize()
        tb = b.tensors[0]
        eco.eco_dequantize(tb.weights, tb.scales, n, 0, 128, 0, deq)
        implicit_master = deq + tb.aux
        torch.testing.assert_close(implicit_master, a.tensors[0].aux, rtol=0, atol=1e-5)
        same = (a.tensors[0].weights == tb.weights).float().mean().item()
        assert same > 0.99, same
    a.close()
    b.close()


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
@pytest.mark.parametrize("bs", [32, 64, 256, 512])
def test_block_sizes(harness, o32, fmt, bs):
    wl = small_mixed_workload(fmt, block_size=bs)
    worst = _run_with_layout(harness, o32, wl, 3, {})
    assert worst["code_mismatch"] == 0, worst


def wide_group_workload(fmt="fp8", **kw):
    """Row-wise and tensor-wise scale groups (the paper's own granularities, Sec. 4.1 and 4.4) of many shapes:
    rows from 8 to 8192 elements (1 to 16 waves per group), ragged last rows, one-scale tensors that fit one
    workgroup and ones that need the two-pass kernels (with and without a ragged last tile)."""
    T = workloads.TensorSpec
    rows = [(5, 1152), (3, 6912), (2, 8192), (7, 520), (9, 96), (4, 1000), (33, 8), (6, 1024), (3, 4096), (2, 5000),
            # rows of which 2, 4 or 8 fill a whole number of waves: a workgroup takes such a bundle (and 5 rows of 1408 do not)
            (8, 1408), (16, 576), (6, 768), (4, 640), (12, 2304), (8, 1152), (5, 1408), (2, 7936)]
    ts = [T(f"row{i}", s, fmt, grad_std=1e-3 * (1 + i % 3), granularity="row") for i, s in enumerate(rows)]
    ts.append(T("row_block_mix", (16, 256), fmt, granularity="row"))            # a row that is also a block size
    ts += [T("tw_small", (4096,), fmt, granularity="tensor"), T("tw_8", (8,), fmt, granularity="tensor"),
           T("tw_big", (300, 1024), fmt, granularity="tensor"), T("tw_ragged", (100003,), fmt, granularity="tensor"),
           T("tw_odd_small", (1001,), fmt, granularity="tensor")]
    ts.insert(4, T("blk", (3000,), fmt))                                          # ordinary block-128 tensor in the same plan
    ts.insert(9, T("norm", (640,), "bf16_plain"))
    return workloads.Workload("wide_" + fmt, ts, steps=3, **kw)


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
@pytest.mark.parametrize("over", [dict(), dict(opt=1, round=1, lr=0.05), dict(mode=3), dict(opt=1, mode=2, lr=0.05),
                                  dict(inject=False, weight_decay=0.1)])
def test_row_wise_and_tensor_wise_groups(harness, o32, fmt, over):
    worst = _run_with_layout(harness, o32, wide_group_workload(fmt), 3, over)
    assert worst["code_mismatch"] == 0, worst


def test_row_wise_bf16_state_and_scales(harness, o32):
    worst = _run_with_layout(harness, o32, wide_group_workload("int4", state_bf16=True, scale_bf16=True, lr=1e-4), 3, {})
    assert worst["code_mismatch"] == 0, worst


def test_initial_quantization_of_wide_groups(harness, eco, o32):
    wl = wide_group_workload("fp8")
    dw = harness.DeviceWorkload(wl, DEV)
    for tv in dw.tensors:
        if tv.scales is None:
            continue
        w0 = workloads.initial_weights(wl, tv.tensor_id, device=DEV).cpu().numpy()
        rc, rs = o32.quantize_rtn(FMT_E4M3, w0, dw.group_size(tv))
        assert np.array_equal(tv.weights.cpu().numpy(), rc), tv.spec.name
        assert np.array_equal(to_f32(tv.scales).view(np.uint32), rs.view(np.uint32)), tv.spec.name
        out = torch.zeros(tv.spec.numel, device=DEV)
        eco.eco_dequantize(tv.weights, tv.scales, tv.spec.numel, 0, dw.group_size(tv), 0, out)
        ref = o32.dequantize(FMT_E4M3, rc, rs, tv.spec.numel, dw.group_size(tv))
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), tv.spec.name
    dw.close()


def test_unsupported_group_sizes_are_rejected(harness, eco):
    n = 20000
    z = torch.zeros(n, device=DEV)
    c = torch.zeros(n, dtype=torch.uint8, device=DEV)
    g = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    for gs in (100, 12, 1004, 9000):
        t = eco.make_tensor(c, z, g, z, z, n, 0, 0, group_size=gs)
        with pytest.raises(eco.EcoError) as ei:
            eco.eco_plan_create([t], eco.make_hparams())
        assert ei.value.status == eco.ECO_EUNSUPPORTED, gs


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
def test_bf16_state_and_scales(harness, o32, fmt):
    wl = small_mixed_workload(fmt, state_bf16=True, scale_bf16=True, lr=1e-4)
    worst = _run_with_layout(harness, o32, wl, 4, {})
    assert worst["code_mismatch"] == 0, worst


def test_identity_format_is_plain_adam(harness, eco, o32):
    """ECO_FMT_FP32_IDENTITY on the device against torch's own Adam (the library comparator of the oracle's pin)."""
    n = 5000
    g = torch.Generator().manual_seed(3)
    w0 = torch.randn(n, generator=g) * 0.02
    w = w0.to(DEV).clone()
    m = torch.zeros(n, device=DEV)
    v = torch.zeros(n, device=DEV)
    grad = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    p = torch.nn.Parameter(w0.double().clone())
    opt = torch.optim.Adam([p], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    t = eco.make_tensor(w, None, grad, m, v, n, 0, eco.ECO_FMT_FP32_IDENTITY)
    with eco.Plan([t], eco.make_hparams()) as plan:
        for k in range(1, 11):
            gk = (torch.randn(n, generator=g) * 1e-3).to(torch.bfloat16)
            grad.copy_(gk)
            p.grad = gk.double()
            opt.step()
            plan.step(eco.make_hparams(step=k))
    torch.cuda.synchronize()
    np.testing.assert_allclose(w.cpu().numpy(), p.detach().numpy(), rtol=2e-5, atol=1e-8)
    np.testing.assert_allclose(m.cpu().numpy(), opt.state[p]["exp_avg"].numpy(), rtol=2e-5, atol=1e-9)
    np.testing.assert_allclose(v.cpu().numpy(), opt.state[p]["exp_avg_sq"].numpy(), rtol=2e-5, atol=1e-14)


# ---------------------------------------------------------------------------------- invariances and edge cases

def _snapshot(dw):
    return [(tv.weights.clone(), None if tv.scales is None else tv.scales.clone(), tv.m.clone(), tv.v.clone())
            for tv in dw.tensors]


def _equal(a, b):
    return all(all((x is None and y is None) or torch.equal(x, y) for x, y in zip(ta, tb)) for ta, tb in zip(a, b))


def test_plans_of_their_own_may_step_concurrently_on_two_streams(harness, eco):
    """eco_step keeps no state outside its plan: two plans (each with block-scaled, row-wise and tensor-wise tensors, so
    each with abs-max scratch of its own) stepped at the same time on two streams give what they give one after the
    other.  Larger tensors than elsewhere in this file, so that the launches of the two streams do overlap."""
    T = workloads.TensorSpec
    def wl(name, fmt):
        ts = [T("blocks", (512, 2048), fmt), T("ragged", (300001,), fmt), T("rows", (300, 2048), fmt, granularity="row"),
              T("whole", (5 * 65536 + 7 * 8,), fmt, granularity="tensor"), T("whole_small", (4096,), fmt, granularity="tensor"),
              T("norm", (2048,), "bf16_plain")]
        return workloads.Workload(name, ts, steps=3)
    results = {}
    for mode in ("serial", "concurrent"):
        a = harness.DeviceWorkload(wl("two_streams_a", "fp8"), DEV)
        b = harness.DeviceWorkload(wl("two_streams_b", "int4"), DEV)
        for k in (1, 2, 3):
            a.fill_gradients(k)
            b.fill_gradients(k)
            torch.cuda.synchronize()
            if mode == "serial":
                a.step(k)
                torch.cuda.synchronize()
                b.step(k)
            else:
                s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
                with torch.cuda.stream(s1):
                    a.step(k)
                with torch.cuda.stream(s2):
                    b.step(k)
            torch.cuda.synchronize()
        results[mode] = (_snapshot(a), _snapshot(b))
        a.close()
        b.close()
    assert _equal(results["serial"][0], results["concurrent"][0]) and _equal(results["serial"][1], results["concurrent"][1])


def test_results_do_not_depend_on_launch_geometry_or_plan_order(harness, eco):
    wl = small_mixed_workload("fp8")
    results = []
    for wgs, reverse in ((0, False), (1, False), (3, True)):
        eco.eco_set_option(0, wgs)
        dw = harness.DeviceWorkload(wl, DEV)
        if reverse:
            dw.plan.close()
            dw.plan = eco.Plan([dw.descriptor(tv) for tv in reversed(dw.tensors)], dw.hparams(1))
        for k in (1, 2, 3):
            dw.fill_gradients(k)
            dw.step(k)
        torch.cuda.synchronize()
        results.append(_snapshot(dw))
        dw.close()
    eco.eco_set_option(0, 0)
    assert _equal(results[0], results[1]) and _equal(results[0], results[2])


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
def test_a_step_launched_in_chunks_gives_the_same_results(harness, eco, fmt):
    """A launch may hold fewer than 2^32 threads, so very large plans are stepped in several launches per kernel
    (and the full-tile kernel loops).  A small limit set from the host makes a small plan take that path: every
    class of scale group, ragged tails and unquantized tensors, several tensor-wise tensors of several tiles."""
    T = workloads.TensorSpec
    ts = [T("blocks", (96, 1024), fmt), T("ragged_a", (4097,), fmt), T("ragged_b", (12345,), fmt), T("ragged_c", (100,), fmt),
          T("rows_2w", (40, 1000), fmt, granularity="row"), T("rows_4w", (37, 2048), fmt, granularity="row"),
          T("rows_16w", (9, 8192), fmt, granularity="row"), T("whole_a", (70000,), fmt, granularity="tensor"),
          T("whole_b", (8193,), fmt, granularity="tensor"), T("whole_c", (3 * 65536,), fmt, granularity="tensor"),
          T("norm", (5000,), "bf16_plain"), T("norm_b", (700,), "bf16_plain"), T("norm_c", (513,), "bf16_plain")]
    wl = workloads.Workload("chunks_" + fmt, ts, steps=3)
    results = []
    for limit in (-1, 1024, 2048 + 1024):
        eco.eco_set_option(3, limit)
        try:
            dw = harness.DeviceWorkload(wl, DEV)
            for k in (1, 2, 3):
                dw.fill_gradients(k)
                dw.step(k)
            torch.cuda.synchronize()
            results.append(_snapshot(dw))
            dw.close()
        finally:
            eco.eco_set_option(3, -1)
    assert _equal(results[0], results[1]) and _equal(results[0], results[2])


def _random_plan(rng, fmt):
    """A random tensor list for one plan: awkward and boundary sizes, every class of scale group."""
    T = workloads.TensorSpec
    ts = []
    for i in range(int(rng.integers(1, 7))):
        kind = rng.choice(["block", "row", "tensor", "plain"], p=[0.4, 0.3, 0.2, 0.1])
        if kind == "row":
            cols = int(rng.choice([8, 24, 96, 128, 512, 520, 576, 640, 768, 1000, 1024, 1408, 2048, 2304, 4096, 4104, 8184, 8192]))
            shape = (int(rng.integers(1, 9)), cols)
        else:
            n = int(rng.choice([1, 7, 8, 127, 128, 511, 512, 513, 4095, 4096, 8191, 8192, 8193, 8200, 20000,
                                int(rng.integers(1, 60000))]))
            shape = (n,)
        if kind == "plain":
            ts.append(T(f"p{i}", shape, "bf16_plain"))
        else:
            ts.append(T(f"{kind}{i}", shape, fmt, grad_std=float(10.0 ** rng.uniform(-4, -2)), granularity=kind))
    return ts


@pytest.mark.parametrize("seed", range(96))
def test_randomized_plans(harness, eco, o32, seed):
    """Seeded random plans: random tensor lists (block, row-wise and tensor-wise groups mixed), block size,
    state and scale types, optimizer, mode, rounding and decay; two steps each, every tensor against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    fmt = "fp8" if rng.random() < 0.5 else "int4"
    opt = int(rng.integers(0, 2))
    mode = int(rng.choice([eco.ECO_MODE_NAIVE, eco.ECO_MODE_ECO, eco.ECO_MODE_MASTER] + ([eco.ECO_MODE_EXACT] if opt == 1 else [])))
    over = dict(opt=opt, mode=mode, round=int(rng.integers(0, 2)), weight_decay=float(rng.choice([0.0, 0.05])),
                lr=float(rng.choice([1e-3, 3e-2])), beta1=float(rng.choice([0.9, 0.5])), seed=int(rng.integers(0, 2 ** 63)))
    wl = workloads.Workload(f"rand{seed}", _random_plan(rng, fmt), steps=2, block_size=int(rng.choice([32, 64, 128, 256, 512])),
                            state_bf16=bool(rng.integers(0, 2)), scale_bf16=bool(rng.integers(0, 2)))
    worst = _run_with_layout(harness, o32, wl, 2, over)
    assert worst.get("code_mismatch", 0) == 0 and worst.get("aux_bit_mismatch", 0) == 0, (worst, over, wl)


def test_results_do_not_depend_on_where_the_arenas_lie(harness, eco):
    """The spread placement (one allocation, arena groups tens of GiB apart) and resident gradient sets (one plan
    per set over the same weights and state) are layout only: same bytes as separate allocations and one set."""
    wl = small_mixed_workload("fp8")
    a = harness.DeviceWorkload(wl, DEV, placement="packed")
    b = harness.DeviceWorkload(wl, DEV, placement="spread", grad_sets=3)
    assert a.placement == "packed" and "GiB apart" in b.placement
    assert b.m.data_ptr() - b.grad.data_ptr() > (20 << 30) and b.v.data_ptr() - b.m.data_ptr() > (20 << 30)
    for k in (1, 2, 3):
        b.fill_gradients(k, k - 1)
    for k in (1, 2, 3):
        a.fill_gradients(k)
        a.step(k)
        b.step(k, k - 1)
    torch.cuda.synchronize()
    assert _equal(_snapshot(a), _snapshot(b))
    # one allocation without gaps, m first and v last, and the plain order
    # ... and the order a bandwidth probe picks at set-up among the gap-free ones (what "auto" chooses for large workloads)
    for placement, first in (("dense", "m"), ("dense-default", "codes"), ("probed", None)):
        c = harness.DeviceWorkload(wl, DEV, placement=placement, grad_sets=2)
        assert "no gaps" in c.placement
        ptrs = {k: getattr(c, k).data_ptr() for k in ("m", "codes", "scales", "grad", "v")}
        if first is not None:
            assert min(ptrs, key=ptrs.get) == first and max(ptrs, key=ptrs.get) == "v"
        else:
            assert "probe" in c.placement and len(c.probe_results) == 5 and all(r["probe_gbs"] > 0 for r in c.probe_results)
        assert ptrs["v"] + c.v.numel() * 4 - min(ptrs.values()) < 2 * harness.DeviceWorkload.pool_bytes(wl, grad_sets=2)
        for k in (1, 2, 3):
            c.fill_gradients(k, k & 1)
            c.step(k, k & 1)
        torch.cuda.synchronize()
        assert _equal(_snapshot(a), _snapshot(c))
        c.close()
    a.close()
    b.close()


@pytest.mark.parametrize("which", ["blocks", "wide_and_tensorwise"])
def test_step_can_be_captured_in_a_hip_graph(harness, eco, which):
    """eco_step allocates nothing, never synchronizes and clears no memory with memset nodes, so a stream
    capture records it (all its kernels, the tensor-wise scratch passes included).  Each replay is one more
    step with the captured hyper-parameters; every replay is compared with the same step issued eagerly,
    with eager work and synchronizations between the replays."""
    wl = small_mixed_workload("fp8") if which == "blocks" else wide_group_workload("fp8")
    a = harness.DeviceWorkload(wl, DEV)
    b = harness.DeviceWorkload(wl, DEV)
    a.fill_gradients(1)
    b.fill_gradients(1)
    b.step(1)                                   # warm-up outside the capture (loads the code objects)
    a.step(1)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        b.step(1)
    torch.cuda.synchronize()
    assert _equal(_snapshot(a), _snapshot(b))   # capturing executed nothing
    scratch = torch.zeros(1 << 20, device=DEV)
    for _ in range(3):
        graph.replay()
        a.step(1)
        torch.cuda.synchronize()
        assert _equal(_snapshot(a), _snapshot(b))
        scratch.add_(1.0)                       # unrelated eager work between the replays
        torch.cuda.synchronize()
    a.close()
    b.close()


def test_plan_less_entry_point_and_resume(harness, eco):
    """eco_step_tensors gives the same bytes as a plan; and because the state is only (codes, scales,
    m, v) plus (seed, step), stopping after 2 steps and continuing equals 4 steps in a row."""
    wl = small_mixed_workload("fp8")
    a = harness.DeviceWorkload(wl, DEV)
    b = harness.DeviceWorkload(wl, DEV)
    for k in (1, 2, 3, 4):
        a.fill_gradients(k)
        a.step(k)
    for k in (1, 2):
        b.fill_gradients(k)
        eco.eco_step_tensors([b.descriptor(tv) for tv in b.tensors], b.hparams(k))
    saved = _snapshot(b)
    c = harness.DeviceWorkload(wl, DEV, init=False)
    for tv, (w, s, m, v) in zip(c.tensors, saved):
        tv.weights.copy_(w)
        if s is not None:
            tv.scales.copy_(s)
        tv.m.copy_(m)
        tv.v.copy_(v)
    for k in (3, 4):
        c.fill_gradients(k)
        c.step(k)
    torch.cuda.synchronize()
    assert _equal(_snapshot(a), _snapshot(c))
    for d in (a, b, c):
        d.close()


def test_zero_gradient_and_zero_blocks(harness, eco, o32):
    """Inactive experts still take the full step (Adam with g = 0 is not a no-op); all-zero weights with
    zero gradient stay zero with scale 0."""
    n = 2048 * 2 + 300
    g = torch.Generator().manual_seed(8)
    w0 = torch.randn(n, generator=g) * 0.02
    w0[:256] = 0.0
    codes = torch.zeros(n, dtype=torch.uint8, device=DEV)
    scales = torch.zeros((n + 127) // 128, device=DEV)
    eco.eco_quantize_init(w0.to(DEV), 0, n, 0, 128, 0, codes, scales)
    m = (torch.randn(n, generator=g) * 1e-4).to(DEV)
    m[:256] = 0.0
    v = (torch.rand(n, generator=g) * 1e-8).to(DEV)
    grad = torch.zeros(n, dtype=torch.bfloat16, device=DEV)

    class TV:
        pass
    tv = TV()
    tv.weights, tv.scales, tv.grad, tv.m, tv.v = codes, scales, grad, m, v
    h = host_copy(tv)
    hp = eco.make_hparams(step=5, seed=77)
    eco.eco_step_tensors([eco.make_tensor(codes, scales, grad, m, v, n, 9, 0)], hp)
    oracle_step(o32, h, n, step_config(hp, 9, 0))
    st = compare(host_copy(tv), h, "zero gradient")
    assert st["code_mismatch"] == 0
    assert torch.all(codes[:256] == 0) and torch.all(scales[:2] == 0) and torch.all(m[:256] == 0)
    assert not torch.equal(m[256:], torch.zeros_like(m[256:]))


def test_step_rejects_a_layout_that_differs_from_the_plan(harness, eco):
    wl = workloads.Workload("tiny", [workloads.TensorSpec("w", (4096,))], steps=1)
    dw = harness.DeviceWorkload(wl, DEV)
    for over in (dict(block_size=64), dict(state_dtype=1), dict(scale_dtype=1), dict(opt=1), dict(mode=0)):
        with pytest.raises(eco.EcoError) as ei:
            dw.plan.step(dw.hparams(1, **over))
        assert ei.value.status == eco.ECO_EINVAL
    with pytest.raises(eco.EcoError):
        dw.plan.step(dw.hparams(0))
    dw.close()
