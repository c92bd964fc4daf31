"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (one plan over every tensor, default launch options).  The step is local to a scale block, so
the oracle recomputes sampled spans of blocks one by one from the inputs the device had before the
step: spans at the start, at a random interior block and at the end of a sample of tensors that
always includes the first and last tensor, a router, the embedding and experts with all-zero
gradients.  Properties that hold at any size are checked on the whole arena."""
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


def pick_spans(wl, rng, n_tensors):
    ids = {0, len(wl.tensors) - 1}
    ids |= {i for i, t in enumerate(wl.tensors) if "router" in t.name or "embed" in t.name and t.fmt != "bf16_plain"}
    ids = set(sorted(ids)[:6]) | {len(wl.tensors) - 1}
    quant = [i for i, t in enumerate(wl.tensors) if t.fmt in ("fp8", "int4")]
    ids |= set(int(x) for x in rng.choice(quant, size=min(n_tensors, len(quant)), replace=False))
    spans = []
    bs = wl.block_size
    for i in sorted(ids):
        t = wl.tensors[i]
        if t.fmt not in ("fp8", "int4"):
            continue
        nb = (t.numel + bs - 1) // bs
        starts = {0, max(0, nb - SPAN_BLOCKS)}
        if nb > 2 * SPAN_BLOCKS:
            starts.add(int(rng.integers(1, nb - SPAN_BLOCKS)))
        for b0 in sorted(starts):
            n = min(SPAN_BLOCKS, nb - b0)
            spans.append((i, b0, n))
    return spans


def grab(tv, wl, b0, nblocks):
    """Host copy of blocks [b0, b0+nblocks) of one tensor."""
    bs = wl.block_size
    e0, e1 = b0 * bs, min((b0 + nblocks) * bs, tv.spec.numel)
    if tv.fmt == 0:
        codes = tv.weights[e0:e1]
    else:
        codes = tv.weights[e0 // 2:(e1 + 1) // 2]
    return dict(codes=codes.cpu().numpy().copy(), scales=to_f32(tv.scales[b0:b0 + nblocks]),
                grad=bf16_bits(tv.grad[e0:e1]), m=to_f32(tv.m[e0:e1]), v=to_f32(tv.v[e0:e1])), e1 - e0


def run_fullsize(wl, steps, n_tensors, seed):
    from paper_2601_22101_amd import harness
    o32 = oracle.get("f32")
    rng = np.random.default_rng(seed)
    dw = harness.DeviceWorkload(wl, DEV)
    total_checked = 0
    mism = 0
    for k in range(1, steps + 1):
        dw.fill_gradients(k)
        spans = pick_spans(wl, rng, n_tensors)
        before = [grab(dw.tensors[i], wl, b0, n) for i, b0, n in spans]
        hp = dw.hparams(k)
        dw.plan.step(hp)
        torch.cuda.synchronize()
        for (i, b0, n), (h, numel) in zip(spans, before):
            tv = dw.tensors[i]
            oracle_step(o32, h, numel, step_config(hp, tv.tensor_id, tv.fmt, elem_offset=b0 * wl.block_size))  # block-128 workloads
            after, _ = grab(tv, wl, b0, n)
            after["grad"] = h["grad"]
            st = compare(after, h, f"{wl.name} step {k} {tv.spec.name} blocks {b0}+{n}", wl.state_bf16)
            mism += st["code_mismatch"]
            total_checked += numel
        # whole-arena properties: every stored value finite, v non-negative, inactive experts still moved
        assert torch.isfinite(dw.m.float().sum()) and torch.isfinite(dw.v.float().sum())
        assert float(dw.v.min()) >= 0.0
    if wl.n_inactive:
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
    assert n > 500_000


def test_config4_smoe_shaped_sampled():
    n = run_fullsize(workloads.config4(), steps=5, n_tensors=24, seed=4)
    assert n > 1_000_000


def test_config5_deepseek_shaped_int4_sampled():
    n = run_fullsize(workloads.config5(), steps=3, n_tensors=24, seed=5)
    assert n > 1_000_000
