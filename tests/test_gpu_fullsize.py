"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (one plan over every tensor, default launch options).  The step is local to a scale block, so
the oracle recomputes sampled spans of blocks one by one from the inputs the device had before the
step: spans at the start, at a random interior block and at the end of a sample of tensors that
always includes the first and last tensor, a router, the embedding and experts with all-zero
gradients -- and, in one step of every run, the first and the last span of EVERY quantized tensor, so
that a wrong entry of the tile -> tensor tables cannot hide in a tensor that was not drawn.
Properties that hold at any size are checked on the whole arena."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from oracle import StepConfig

from gpu_util import ORACLE_FMT, bf16_bits, compare, oracle_step, step_config, to_f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SPAN_BLOCKS = 48          # 6144 elements: twelve 512-element tiles, not tile aligned in general
EDGE_BLOCKS = 24          # spans of the every-tensor sweep: 3072 elements at each end of each tensor


def pick_spans(wl, rng, n_tensors):
    """(tensor, first group, number of groups) samples; groups are the tensor's own scale groups (blocks,
    rows, or the whole tensor), spans hold about SPAN_BLOCKS * 128 elements."""
    ids = {0, len(wl.tensors) - 1}
    ids |= {i for i, t in enumerate(wl.tensors) if "router" in t.name or "embed" in t.name and t.fmt != "bf16_plain"}
    ids = set(sorted(ids)[:6]) | {len(wl.tensors) - 1}
    quant = [i for i, t in enumerate(wl.tensors) if t.fmt in ("fp8", "int4")]
    ids |= set(int(x) for x in rng.choice(quant, size=min(n_tensors, len(quant)), replace=False))
    spans = []
    for i in sorted(ids):
        t = wl.tensors[i]
        if t.fmt not in ("fp8", "int4"):
            continue
        gs = t.group_size(wl.block_size)
        ng = (t.numel + gs - 1) // gs
        per = max(1, SPAN_BLOCKS * 128 // gs)
        starts = {0, max(0, ng - per)}
        if ng > 2 * per:
            starts.add(int(rng.integers(1, ng - per)))
        for g0 in sorted(starts):
            spans.append((i, g0, min(per, ng - g0)))
    return spans


def edge_spans(wl):
    """First and last span of every quantized tensor (one span when the tensor is short)."""
    spans = []
    for i, t in enumerate(wl.tensors):
        if t.fmt not in ("fp8", "int4"):
            continue
        gs = t.group_size(wl.block_size)
        ng = (t.numel + gs - 1) // gs
        per = max(1, EDGE_BLOCKS * 128 // gs)
        if gs >= t.numel and t.numel > 1 << 17:
            continue              # one scale over a large tensor: the span would be the whole tensor (sampled instead)
        for g0 in sorted({0, max(0, ng - per)}):
            spans.append((i, g0, min(per, ng - g0)))
    return spans


def grab(tv, wl, g0, ngroups, with_aux=False):
    """Host copy of scale groups [g0, g0+ngroups) of one tensor."""
    gs = tv.spec.group_size(wl.block_size)
    e0, e1 = g0 * gs, min((g0 + ngroups) * gs, tv.spec.numel)
    assert e0 % 2 == 0
    if tv.fmt == 0:
        codes = tv.weights[e0:e1]
    else:
        codes = tv.weights[e0 // 2:(e1 + 1) // 2]
    h = dict(codes=codes.cpu().numpy().copy(), scales=to_f32(tv.scales[g0:g0 + ngroups]),
             grad=bf16_bits(tv.grad[e0:e1]), m=to_f32(tv.m[e0:e1]), v=to_f32(tv.v[e0:e1]))
    if with_aux:
        h["aux"] = to_f32(tv.aux[e0:e1])
    return h, e1 - e0


def all_finite(arena):
    """Every element of a (possibly bf16) device arena is finite; chunked to keep the fp32 temporaries small."""
    return all(bool(torch.isfinite(c.float().sum())) for c in arena.split(1 << 28))


def run_fullsize(wl, steps, n_tensors, seed, layout=None, every_tensor_step=2):
    from paper_2601_22101_amd import harness
    o32 = oracle.get("f32")
    rng = np.random.default_rng(seed)
    dw = harness.DeviceWorkload(wl, DEV, layout=layout)
    with_aux = dw.aux is not None
    total_checked = 0
    mism = 0
    for k in range(1, steps + 1):
        dw.fill_gradients(k)
        spans = pick_spans(wl, rng, n_tensors)
        if k == min(every_tensor_step, steps):
            have = {(i, g0) for i, g0, _ in spans}
            spans += [sp for sp in edge_spans(wl) if (sp[0], sp[1]) not in have]
        print(f"[fullsize] {wl.name} step {k}: {len(spans)} spans", flush=True)
        before = [grab(dw.tensors[i], wl, g0, n, with_aux) for i, g0, n in spans]
        hp = dw.hparams(k)
        dw.plan.step(hp)
        torch.cuda.synchronize()
        for (i, g0, n), (h, numel) in zip(spans, before):
            tv = dw.tensors[i]
            gs = tv.spec.group_size(wl.block_size)
            oracle_step(o32, h, numel, step_config(hp, tv.tensor_id, tv.fmt, elem_offset=g0 * gs, group_size=gs))
            after, _ = grab(tv, wl, g0, n, with_aux)
            after["grad"] = h["grad"]
            st = compare(after, h, f"{wl.name} step {k} {tv.spec.name} groups {g0}+{n}", wl.state_bf16)
            mism += st["code_mismatch"]
            total_checked += numel
        # whole-arena properties: every stored value finite, v non-negative, inactive experts still moved
        assert all_finite(dw.m) and all_finite(dw.v)
        assert float(dw.v.min()) >= 0.0
    if wl.n_inactive and dw.hparams(1).opt == 0:
        # an expert that never received a gradient keeps m = v = 0 only if it was inactive at every step;
        # one that was inactive at the last step but active before must still have had its state stepped
        last = steps
        for tv in dw.tensors:
            t = tv.spec
            if t.expert >= 0 and t.expert in workloads.inactive_experts(wl, last, t.layer):
                was_active = any(t.expert not in workloads.inactive_experts(wl, s, t.layer) for s in range(1, last))
                if was_active:
                    assert float(tv.v.float().abs().max()) > 0
                    assert float(tv.grad.float().abs().max()) == 0
                    break
    dw.close()
    assert mism == 0
    return total_checked


def test_config3_gemma_shaped_sampled():
    n = run_fullsize(workloads.config3(), steps=5, n_tensors=10, seed=3)
    assert n > 1_500_000


def test_config4_smoe_shaped_sampled():
    n = run_fullsize(workloads.config4(), steps=5, n_tensors=24, seed=4)
    assert n > 19_000_000          # 3 153 tensors x two spans of 3 072 elements, plus the sampled spans


def test_config5_deepseek_shaped_int4_sampled():
    n = run_fullsize(workloads.config5(), steps=3, n_tensors=24, seed=5)
    assert n > 34_000_000          # 5 685 tensors x two spans


def test_config4_row_wise_sampled():
    """One scale per row (Sec. 4.1): the wide-group kernel at full size; spans are whole rows."""
    n = run_fullsize(workloads.with_granularity(workloads.config4(), "row"), steps=3, n_tensors=16, seed=14)
    assert n > 300_000


def test_config5_row_wise_int4_sampled():
    """One scale per row on the INT4 / bf16-state set: the wide-group kernel with rows of 1408 and 2048 elements."""
    n = run_fullsize(workloads.with_granularity(workloads.config5(), "row"), steps=2, n_tensors=16, seed=18)
    assert n > 20_000_000


def test_config6_paper_shapes_row_wise_sampled():
    """The paper's own SMoE shapes with its FP8 granularity: rows of 576 and 2304 elements, which the wide-group kernel
    steps eight and two to a workgroup; unquantized attention, router and embedding in the same plan."""
    n = run_fullsize(workloads.with_granularity(workloads.config6(), "row"), steps=2, n_tensors=16, seed=19)
    assert n > 8_000_000          # 1 536 expert matrices x two spans of five rows of 576 or one row of 2304 elements


def test_config4_tensor_wise_sampled():
    """One scale per tensor (Sec. 4.4): the two-pass kernels at full size; every sampled tensor is recomputed whole
    (the embedding of 51.5 M elements and the 65 536-element router included)."""
    n = run_fullsize(workloads.with_granularity(workloads.config4(), "tensor"), steps=2, n_tensors=6, seed=15)
    assert n > 50_000_000


def test_config5_tensor_wise_int4_sampled():
    """The paper's INT4 setting (tensor-wise scales) on the DeepSeek-shaped set with bf16 state and scales."""
    n = run_fullsize(workloads.with_granularity(workloads.config5(), "tensor"), steps=2, n_tensors=4, seed=16)
    assert n > 100_000_000


@pytest.mark.parametrize("variant", ["adam-master", "sgdm-eco", "sgdm-exact"])
def test_config4_other_modes_sampled(variant):
    from paper_2601_22101_amd import binding as eco
    layout = {"adam-master": dict(mode=eco.ECO_MODE_MASTER),
              "sgdm-eco": dict(opt=eco.ECO_OPT_SGDM),
              "sgdm-exact": dict(opt=eco.ECO_OPT_SGDM, mode=eco.ECO_MODE_EXACT)}[variant]
    n = run_fullsize(workloads.config4(), steps=2, n_tensors=12, seed=17, layout=layout)
    assert n > 300_000


# ------------------------------------------------------------------ one tensor at the largest sizes
CHUNK = 1 << 28


def _one_huge_tensor(eco, o32, numel, fmt, state_bf16, span_edges, seed):
    """One block-scaled tensor of `numel` elements, set up chunk by chunk (the initial quantizer is local to a
    scale block, so quantizing slices of whole blocks is quantizing the tensor), stepped once through the
    plan-less entry point; the oracle recomputes the spans [e0, e1) from the inputs the device held."""
    sdt = torch.bfloat16 if state_bf16 else torch.float32
    dt = eco.ECO_DT_BF16 if state_bf16 else eco.ECO_DT_FP32
    need = numel * ((1 if fmt == 0 else 0.5) + 2 + 2 * (2 if state_bf16 else 4)) + numel // 128 * 4 + (6 << 30)
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < need:
        pytest.skip(f"needs {need / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB are free")
    codes = torch.empty(numel if fmt == 0 else numel // 2, dtype=torch.uint8, device=DEV)
    scales = torch.empty((numel + 127) // 128, dtype=sdt, device=DEV)
    grad = torch.empty(numel, dtype=torch.bfloat16, device=DEV)
    m = torch.empty(numel, dtype=sdt, device=DEV)
    v = torch.empty(numel, dtype=sdt, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    for off in range(0, numel, CHUNK):
        n = min(CHUNK, numel - off)
        src = torch.randn(n, device=DEV, generator=gen) * 0.02
        eco.eco_quantize_init(src, eco.ECO_DT_FP32, n, fmt, 128, dt, codes[off if fmt == 0 else off // 2:], scales[off // 128:])
        m[off:off + n] = (torch.randn(n, device=DEV, generator=gen) * 1e-3).to(sdt)
        v[off:off + n] = (torch.rand(n, device=DEV, generator=gen) * 1e-5).to(sdt)
        grad[off:off + n] = (torch.randn(n, device=DEV, generator=gen) * 2e-3).to(torch.bfloat16)
        torch.cuda.synchronize()
        del src
        if off % (16 * CHUNK) == 0:
            print(f"[huge] filled {off + n} of {numel}", flush=True)

    def grab(e0, e1):
        c = codes[e0:e1] if fmt == 0 else codes[e0 // 2:(e1 + 1) // 2]
        return dict(codes=c.cpu().numpy().copy(), scales=to_f32(scales[e0 // 128:(e1 + 127) // 128]), grad=bf16_bits(grad[e0:e1]),
                    m=to_f32(m[e0:e1]), v=to_f32(v[e0:e1]))

    hp = eco.make_hparams(block_size=128, state_dtype=dt, scale_dtype=dt, lr=1e-3, step=3, seed=seed)
    before = [grab(e0, e1) for e0, e1 in span_edges]
    print(f"[huge] stepping {numel} elements", flush=True)
    eco.eco_step_tensors([eco.make_tensor(codes, scales, grad, m, v, numel, 11, fmt)], hp)
    torch.cuda.synchronize()
    for (e0, e1), h in zip(span_edges, before):
        oracle_step(o32, h, e1 - e0, step_config(hp, 11, fmt, elem_offset=e0, group_size=128))
        after = grab(e0, e1)
        after["grad"] = h["grad"]
        st = compare(after, h, f"elements [{e0}, {e1}) of {numel}", state_bf16)
        assert st["code_mismatch"] == 0
    assert all_finite(m) and all_finite(v)
    del codes, scales, grad, m, v
    torch.cuda.empty_cache()


def test_one_fp8_tensor_of_more_than_2_pow_32_elements():
    """Element indices beyond 32 bits in the FP8 / fp32-state kernel and its ragged tail."""
    from paper_2601_22101_amd import binding as eco
    n = (1 << 32) + 3 * 512 + 100
    _one_huge_tensor(eco, oracle.get("f32"), n, 0, False,
                     [(0, 6144), ((1 << 31) - 3072, (1 << 31) + 3072), ((1 << 32) - 3072, n)], seed=32)


def test_one_int4_tensor_of_more_than_2_pow_35_elements():
    """The largest plan 288 GB hold (INT4 codes, bf16 scales, gradient and state: 6.5 bytes per element): more tiles than
    one launch can take workgroups, and random-number counters (element index / 8) beyond 32 bits."""
    from paper_2601_22101_amd import binding as eco
    n = (1 << 35) + 3 * 512 + 100
    _one_huge_tensor(eco, oracle.get("f32"), n, 1, True,
                     [(0, 6144), ((1 << 32) - 3072, (1 << 32) + 3072), ((1 << 35) - 3072, n)], seed=35)
