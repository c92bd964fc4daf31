#!/usr/bin/env python3
"""Benchmark of the ECO optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]

A "step" is one eco_step call over the whole synthetic parameter set (dequantize, Adam update without
master weights, abs-max re-quantization with stochastic rounding, error injection into momentum), with
all inputs resident in HBM.  The fresh bf16 gradients of every step are drawn on the device before the
timed region, one gradient arena per step; the K timed steps then run back to back between two
synchronizations.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "ECO optimizer-step params/sec and achieved HBM GB/s (% of peak), 1 GPU"
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, vendor figure

# Algorithmic bytes per parameter the method must move in one step (read + write):
#   FP8 codes 1+1, fp32 scale per 128 elements (4+4)/128, bf16 gradient 2, fp32 m 4+4, fp32 v 4+4
BYTES_PER_PARAM = {"fp8": 20.0625, "int4": 11.03125, "bf16_plain": 22.0}


def algorithmic_bytes(wl, variant: str = "adam-sr") -> float:
    """Bytes the method itself must move in one step (read + write), summed over the tensors.  A tensor
    with a single scale that does not fit one workgroup needs its inputs twice (the abs-max of theta~ must
    be known before any element can be quantized): its reads count double."""
    adam = variant.startswith("adam")
    master = "master" in variant
    exact = "exact" in variant
    total = 0.0
    for t in wl.tensors:
        st = 2 if wl.state_bf16 else 4
        state = (2 if adam else 1) * 2 * st                      # m (and v): read + write
        if t.fmt in ("fp8", "int4"):
            code = 1.0 if t.fmt == "fp8" else 0.5
            sb = (2 if wl.scale_bf16 else 4) / wl.block_size
            gs = t.group_size(wl.block_size)
            sb = (2 if wl.scale_bf16 else 4) / gs
            two_pass = gs >= t.numel and not (t.numel <= 8192 and t.numel % 8 == 0)
            if master:                                             # master read+write, codes and scales written only
                rd, wr = 4 + 2 + state / 2, 4 + code + sb + state / 2
            else:
                rd = code + sb + 2 + state / 2 + (4 if exact else 0)
                wr = code + sb + state / 2 + (4 if exact else 0)
            per = rd * (2 if two_pass else 1) + wr
        else:
            per = 2 * 2 + 2 + state
        total += t.numel * per
    return total


def kernel_source_hash() -> str:
    """sha256 over the library's kernel and launch sources: what a committed profile was measured on."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2601_22101_amd", "csrc")
    for fn in sorted(os.listdir(d)):
        if fn.endswith((".hip", ".hpp", ".cpp")):
            h.update(fn.encode())
            h.update(open(os.path.join(d, fn), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(wl_name: str):
    """HBM bytes per launch from the COMMITTED rocprofv3 --pmc summary of this workload (FETCH_SIZE / WRITE_SIZE scaled
    by a copy of known size); it is not measured in this run.  Returns (bytes or None, where it comes from): None when
    there is no record or when the record was taken on other kernel sources than the ones in the tree."""
    tag = {"cfg4_smoe_2p1b_shaped": "fp8_cfg4"}.get(wl_name)
    if not tag:
        return None, None
    rel = os.path.join("profiles", f"eco_step_kernel_{tag}_hbm_traffic.txt")
    val = src = None
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch="):
                val = float(line.split("=", 1)[1])
            if line.startswith("kernel_source_sha256="):
                src = line.split("=", 1)[1].strip()
    except OSError:
        return None, None
    if val is None:
        return None, None
    if src != kernel_source_hash():
        return None, f"{rel} was taken on kernel sources {src}, the tree holds {kernel_source_hash()}: stale, not reported"
    return val, f"replayed from {rel} (rocprofv3 --pmc on kernel sources {src}); not measured in this run"


def static_bytes_per_param(wl, variant: str) -> float:
    """Bytes of weights + optimizer state resident per parameter (the paper's memory accounting, Sec. 4.2
    "Memory and Runtime": 12 B with fp32 master weights, m and v; 9 B with FP8 weights, m and v)."""
    st = 2 if wl.state_bf16 else 4
    sc = 2 if wl.scale_bf16 else 4
    total = 0.0
    for t in wl.tensors:
        if t.fmt in ("fp8", "int4"):
            b = (1.0 if t.fmt == "fp8" else 0.5) + sc / t.group_size(wl.block_size)
        else:
            b = 2.0
        b += st * (2 if variant.startswith("adam") else 1)
        if "master" in variant or "exact" in variant:
            b += 4.0
        total += b * t.numel
    return total / wl.numel


def cpu_baseline(wl, target_seconds: float = 10.0) -> dict:
    """The CPU oracle, as it stands, timed on a bounded sample of the same workload (host cores of this machine)."""
    import numpy as np

    import oracle
    import workloads

    o = oracle.get("f32")
    fmt_map = {"fp8": oracle.FMT_E4M3, "int4": oracle.FMT_INT4}
    quant = [i for i, t in enumerate(wl.tensors) if t.fmt in fmt_map]

    def prepare(ids):
        items = []
        for i in ids:
            t = wl.tensors[i]
            w = workloads.initial_weights(wl, i, "cpu").numpy()
            codes, scales = o.quantize_rtn(fmt_map[t.fmt], w, wl.block_size, wl.scale_bf16)
            g = workloads.gradient(wl, i, 1, "cpu")
            import torch
            g16 = g.view(torch.int16).numpy().view(np.uint16).copy()
            items.append((i, t, codes, scales, g16, np.zeros(t.numel, np.float32), np.zeros(t.numel, np.float32)))
        return items

    def run(items, step=1):
        n = 0
        t0 = time.perf_counter()
        for i, t, codes, scales, g16, m, v in items:
            cfg = oracle.StepConfig(fmt=fmt_map[t.fmt], block_size=wl.block_size, state_bf16=wl.state_bf16,
                                    scale_bf16=wl.scale_bf16, lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps,
                                    step=step, seed=workloads.BASE_SEED, tensor_id=i)
            assert o.eco_step(cfg, t.numel, m, v, codes=codes, scales=scales, grad_bf16=g16) == 0
            n += t.numel
        return n, time.perf_counter() - t0

    # probe with the first tensor(s) up to ~2M parameters, then size the sample for the time target
    probe_ids, acc = [], 0
    for i in quant:
        probe_ids.append(i)
        acc += wl.tensors[i].numel
        if acc >= 2_000_000:
            break
    n0, dt0 = run(prepare(probe_ids))
    rate = n0 / dt0
    want = min(rate * target_seconds, 6.0e8)          # also bounds the time spent preparing host inputs
    ids, acc = [], 0
    for i in quant:
        if acc >= want and ids:
            break
        if acc + wl.tensors[i].numel > 4 * want and ids:
            continue
        ids.append(i)
        acc += wl.tensors[i].numel
    items = prepare(ids)
    n = dt = 0.0
    steps = 0
    while steps < 8 and (steps == 0 or dt < target_seconds):      # consecutive steps on the same sample
        steps += 1
        n1, dt1 = run(items, steps)
        n += n1
        dt += dt1
    threads = o.num_threads()
    # the same oracle on one thread, on the first tensors of the sample (about two seconds of work)
    o.set_threads(1)
    sub, acc = [], 0
    for it in items:
        sub.append(it)
        acc += it[1].numel
        if acc >= 0.12 * rate * 16 / max(threads, 1):
            break
    n1t, dt1t = run(sub, steps + 1)
    o.set_threads(threads)
    return {"value": n / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
            "single_thread_value": n1t / dt1t, "cpu_model": cpu_model(),
            "sample": f"{steps} consecutive steps over the first {len(ids)} quantized tensors of the workload "
                      f"({int(n1)} parameters each), fp32 build of the oracle, {dt:.1f} s; single thread: one step over "
                      f"{int(n1t)} parameters, {dt1t:.1f} s"}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parity_step(dw, wl, step: int, gset: int, n_tensors: int = 40) -> dict:
    """Part of the CPU-baseline leg: one more, untimed, step of the workload that was just timed, in the same launch
    configuration; the oracle recomputes a seeded sample of block spans (start, interior, end of a sample of tensors that
    includes the first and the last tensor, routers, the embedding) from the inputs the device held before the step, and
    the device's results are compared with it element by element."""
    import numpy as np
    import torch

    import oracle
    o = oracle.get("f32")
    fmt_map = {"fp8": oracle.FMT_E4M3, "int4": oracle.FMT_INT4}
    rng = np.random.default_rng(workloads_seed() + step)
    quant = [i for i, t in enumerate(wl.tensors) if t.fmt in fmt_map]
    ids = {quant[0], quant[-1]} | {i for i in quant if "router" in wl.tensors[i].name or "embed" in wl.tensors[i].name}
    ids = set(sorted(ids)[:8]) | {quant[-1]}
    ids |= set(int(x) for x in rng.choice(quant, size=min(n_tensors, len(quant)), replace=False))
    spans = []
    for i in sorted(ids):
        t = wl.tensors[i]
        gs = t.group_size(wl.block_size)
        ng = (t.numel + gs - 1) // gs
        per = max(1, 48 * 128 // gs)
        if gs >= t.numel and t.numel > 1 << 21:
            continue
        starts = {0, max(0, ng - per)}
        if ng > 2 * per:
            starts.add(int(rng.integers(1, ng - per)))
        spans += [(i, g0, min(per, ng - g0)) for g0 in sorted(starts)]

    def bits16(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()

    def f32(t):
        return oracle.bf16_bits_to_f32(bits16(t)) if t.dtype == torch.bfloat16 else t.cpu().numpy().astype(np.float32)

    def grab(i, g0, n):
        tv = dw.tensors[i]
        gs = tv.spec.group_size(wl.block_size)
        e0, e1 = g0 * gs, min((g0 + n) * gs, tv.spec.numel)
        codes = tv.weights[e0:e1] if tv.spec.fmt == "fp8" else tv.weights[e0 // 2:(e1 + 1) // 2]
        h = dict(codes=codes.cpu().numpy().copy(), scales=f32(tv.scales[g0:g0 + n]), grad=bits16(dw.grad_view(tv, gset)[e0:e1]),
                 m=f32(tv.m[e0:e1]), v=f32(tv.v[e0:e1]))
        if tv.aux is not None:                       # master weights, or the stored error of the exact injection
            h["aux"] = f32(tv.aux[e0:e1])
        return h, e1 - e0

    before = [grab(*sp) for sp in spans]
    hp = dw.hparams(step)
    dw.step(step, gset)
    torch.cuda.synchronize()
    out = {"elements": 0, "spans": len(spans), "tensors": len(ids), "code_mismatches": 0, "scale_mismatches": 0,
           "m_max_rel": 0.0, "v_max_rel": 0.0, "m_bit_mismatches": 0, "v_bit_mismatches": 0}
    for (i, g0, n), (h, numel) in zip(spans, before):
        t = wl.tensors[i]
        gs = t.group_size(wl.block_size)
        cfg = oracle.StepConfig(fmt=fmt_map[t.fmt], opt=hp.opt, round=hp.round, mode=hp.mode, block_size=gs,
                                state_bf16=wl.state_bf16, scale_bf16=wl.scale_bf16, lr=hp.lr, beta1=hp.beta1, beta2=hp.beta2,
                                eps=hp.eps, weight_decay=hp.weight_decay, step=hp.step, seed=hp.seed, elem_offset=g0 * gs,
                                tensor_id=i)
        assert o.eco_step(cfg, numel, h["m"], h["v"] if hp.opt == 0 else None, codes=h["codes"], scales=h["scales"],
                          grad_bf16=h["grad"], aux=h.get("aux")) == 0
        got, _ = grab(i, g0, n)
        if "aux" in h:
            out["aux_bit_mismatches"] = out.get("aux_bit_mismatches", 0) + int((got["aux"].view(np.uint32) != h["aux"].view(np.uint32)).sum())
        out["elements"] += numel
        out["code_mismatches"] += int((got["codes"] != h["codes"]).sum())
        out["scale_mismatches"] += int((got["scales"].view(np.uint32) != h["scales"].view(np.uint32)).sum())
        for key in ("m", "v") if hp.opt == 0 else ("m",):
            a, b = got[key].astype(np.float64), h[key].astype(np.float64)
            rel = np.abs(a - b) / np.maximum(np.abs(b), 1e-30)
            out[f"{key}_max_rel"] = max(out[f"{key}_max_rel"], float(rel.max()))
            out[f"{key}_bit_mismatches"] += int((got[key].view(np.uint32) != h[key].view(np.uint32)).sum())
    out["flip_rate"] = out["code_mismatches"] / max(out["elements"], 1)
    out["what"] = (f"step {step} (one more step after the timed ones, same plan and launch configuration): the oracle recomputed "
                   f"{len(spans)} spans of scale groups of {len(ids)} tensors from the device's inputs")
    return out


def workloads_seed() -> int:
    import workloads
    return workloads.BASE_SEED


def time_launches(fn, reps: int, warm: int = 2):
    """Average / median / min duration (ms) of `reps` calls of fn(), events on the current stream."""
    import torch
    for _ in range(warm):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for i in range(reps):
        ev[i].record()
        fn()
    ev[reps].record()
    torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    return sum(ms) / len(ms), ms[len(ms) // 2], ms[0]


def address_map(torch, workloads, eco, harness) -> int:
    """Where the arrays of the step lie in device memory, and what that does to it.  One allocation of most of the
    device's memory; (1) the library's byte-mix probe (the loads and stores of the FP8 / fp32-state Adam step on 2^30
    elements, no arithmetic) with codes, scales, gradient and m packed at R GiB into the allocation and v moved through it
    in steps of 4 GiB; (2) the step itself on configuration 4 with its arenas packed at the start of the allocation, and
    with only the v arena moved to the start of every 32 GiB region.  Prints the tables; the last line is JSON."""
    GiB, MiB = 1 << 30, 1 << 20
    free = torch.cuda.mem_get_info()[0]
    pool_gib = min(244, int((free - (12 << 30)) // (4 * GiB) * 4))
    pool = torch.zeros(pool_gib * GiB, dtype=torch.uint8, device="cuda:0")
    base = pool.data_ptr()
    numel = 1 << 30
    size = dict(codes=1 * GiB, scales=32 * MiB, grad=2 * GiB, m=4 * GiB, v=4 * GiB)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    def probe(at):
        for k, p in at.items():
            assert 0 <= p and p + size[k] <= pool_gib * GiB, (k, p)
        a = {k: base + p for k, p in at.items()}
        for i in range(4):                        # one warm-up launch, three timed ones; the best counts
            eco.eco_bandwidth_probe(0, a["codes"], a["scales"], a["grad"], a["m"], a["v"], numel)
            ev[i].record()
        torch.cuda.synchronize()
        return numel * BYTES_PER_PARAM["fp8"] / min(ev[i].elapsed_time(ev[i + 1]) for i in range(3)) / 1e6

    print(f"one allocation of {pool_gib} GiB; byte-mix probe on 2^30 elements, GB/s of algorithmic traffic / 10;", flush=True)
    print("codes, scales, gradient, m packed from R GiB on (7 GiB); columns: v at 0, 4, 8, ... GiB ('.' = overlap)", flush=True)
    table = {}
    for R in range(0, pool_gib - 8, 32):
        row = []
        for g in range(0, pool_gib - 4, 4):
            if g < R + 8 and g + 4 > R:
                row.append(None)
                continue
            at = dict(codes=R * GiB, scales=(R + 1) * GiB, grad=(R + 1) * GiB + 32 * MiB, m=(R + 3) * GiB + 32 * MiB, v=g * GiB)
            row.append(probe(at))
        table[R] = row
        print("R=%3d: %s" % (R, " ".join("   ." if x is None else "%4.0f" % (x / 10) for x in row)), flush=True)
    # regions (32 GiB) in which v is slow, for every R: the kinds of region show as identical rows
    slow = {}
    for R, row in table.items():
        vals = [x for x in row if x is not None]
        cut = (min(vals) + max(vals)) / 2
        per_region = {}
        for i, x in enumerate(row):
            if x is not None:
                per_region.setdefault(i * 4 // 32, []).append(x < cut)
        slow[R] = [r for r, flags in sorted(per_region.items()) if sum(flags) * 2 > len(flags)]
        print(f"rest in region {R // 32}: v is slow in regions {slow[R]}", flush=True)

    wl = workloads.CONFIGS[4]()
    steps = {}
    packed_v_gib = None
    for v_gib in [None] + list(range(32, pool_gib - 13, 32)):
        skew = {}
        if v_gib is not None:
            skew["v"] = (int((v_gib - packed_v_gib) * GiB) >> 21) << 21
        dw = harness.DeviceWorkload(wl, "cuda:0", init="bulk", single_allocation=pool, skew_bytes=skew, grad_sets=1)
        dw.fill_gradients_bulk(1, 0)
        torch.cuda.synchronize()
        at = {k: round((getattr(dw, k).data_ptr() - base) / GiB, 1) for k in ("codes", "grad", "m", "v")}
        if v_gib is None:
            packed_v_gib = (dw.v.data_ptr() - base) / GiB
        kk = [0]

        def one():
            kk[0] += 1
            dw.step(kk[0], 0)
        avg, med, mn = time_launches(one, 5, warm=2)
        steps[at["v"]] = med
        print(f"configuration 4, the step itself: codes at {at['codes']}, gradient at {at['grad']}, m at {at['m']}, v at {at['v']} GiB: "
              f"median {med:.3f} ms = {100 * algorithmic_bytes(wl) / med / 1e6 / HBM_PEAK_GBS:.1f} % of peak", flush=True)
        dw.close()
        del dw
    print(json.dumps({"address_map": {"pool_gib": pool_gib, "probe_gbs_by_R_and_v": {str(R): [None if x is None else round(x) for x in row]
                                                                                       for R, row in table.items()},
                                      "slow_regions_of_v_by_R": {str(R): v for R, v in slow.items()},
                                      "step_ms_by_v_gib": steps}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload number: 1-5 = the baseline's configurations; 6 = the shapes of the paper's own SMoE model (Sec. 4.2)")
    ap.add_argument("--wgs-per-cu", type=int, default=0, help="launch tuning: workgroups per compute unit (0 = default)")
    ap.add_argument("--lds-bytes", type=int, default=-1, help="launch tuning: dynamic LDS per workgroup (-1 = default)")
    ap.add_argument("--lds-bytes-wave", type=int, default=-1,
                    help="launch tuning: dynamic LDS per wave of the wide-group and tensor-wise kernels (-1 = default)")
    ap.add_argument("--variant", default="adam-sr",
                    choices=["adam-sr", "adam-rtn", "sgdm-sr", "sgdm-rtn", "adam-naive-sr", "adam-master-sr",
                             "adam-master-rtn", "sgdm-master-sr", "sgdm-exact-sr"],
                    help="optimizer / mode / rounding variant of the step (the headline metric is adam-sr = Adam-ECO "
                         "with stochastic rounding; 'master' is the fp32-master-weight baseline, 'exact' the "
                         "stored-error injection of Appendix A, 'naive' master weights removed without injection)")
    ap.add_argument("--granularity", default="block", choices=["block", "row", "tensor"],
                    help="scale groups of the quantized tensors: the configuration's 128-element blocks (headline), "
                         "one scale per row (the paper's FP8 runs) or per tensor (its INT4 run)")
    ap.add_argument("--placement", default="auto", choices=["auto", "packed", "spread", "dense", "dense-default", "probed"],
                    help="where the harness puts the arenas in HBM: one allocation per arena (packed); one allocation without "
                         "gaps, m first and v last with codes, scales and gradients between them (dense) or in the order codes, "
                         "scales, gradients, m, v (dense-default); one allocation without gaps, m first and v after as many of "
                         "the other arenas as the library's bandwidth probe finds fastest at set-up (probed; auto = probed for "
                         "FP8 / fp32-state Adam workloads of 8 GiB and more, dense for other large ones); one allocation with the "
                         "codes+gradient, m and v arenas tens of GiB of unused memory apart (spread)")
    ap.add_argument("--spread-gap-gib", type=int, default=0, help="distance between the arena groups of the spread placement (0 = default)")
    ap.add_argument("--calibrate-gaps", type=int, default=3,
                    help="spread placement: time this many candidate distances (the default and smaller ones, 8 GiB apart) "
                         "in a probe at set-up and keep the fastest (0 or 1 = use the default distance)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the untimed parity step after the timed region")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the copy-kernel ceilings after the timed region")
    ap.add_argument("--compare-placements", default=None,
                    help="comma-separated placements to time the same step on after the main run (configuration 4 only; "
                         "default: dense,packed,spread for the headline variant, none for the others; empty = none)")
    ap.add_argument("--bulk-grad", action="store_true",
                    help="draw each step's gradients with a few generator calls over the whole arena instead of one "
                         "per tensor (same distribution; for runs under rocprofv3 --pmc)")
    ap.add_argument("--bulk-init", action="store_true",
                    help="write the initial quantized weights with a few launches over the whole arenas (arbitrary valid "
                         "codes and scales instead of quantized N(0, 0.02) draws; for runs under rocprofv3 --pmc)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps, run two plain 1 GiB device copies (a reference of known size for "
                         "scaling rocprofv3 byte counters)")
    ap.add_argument("--address-map", action="store_true",
                    help="instead of the benchmark: time the library's bandwidth probe, and the step itself, with the arrays "
                         "placed by hand in one large allocation, and print where in it they get in each other's way")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build measures the ECO step on ONE GPU only (the step shards over blocks with no "
              "exchange; multi-GPU runs are not part of it). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import workloads
    from paper_2601_22101_amd import binding as eco
    from paper_2601_22101_amd import harness

    if args.address_map:
        return address_map(torch, workloads, eco, harness)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.wgs_per_cu:
        eco.eco_set_option(0, args.wgs_per_cu)
    if args.lds_bytes >= 0:
        eco.eco_set_option(1, args.lds_bytes)
    if args.lds_bytes_wave >= 0:
        eco.eco_set_option(2, args.lds_bytes_wave)

    wl = workloads.CONFIGS[args.config]()
    if args.granularity != "block":
        wl = workloads.with_granularity(wl, args.granularity)
    over = {}
    if args.variant.startswith("sgdm"):
        over["opt"] = eco.ECO_OPT_SGDM
    if args.variant.endswith("rtn"):
        over["round"] = eco.ECO_ROUND_RTN
    if "master" in args.variant:
        over["mode"] = eco.ECO_MODE_MASTER
    elif "exact" in args.variant:
        over["mode"] = eco.ECO_MODE_EXACT
    elif "naive" in args.variant:
        over["mode"] = eco.ECO_MODE_NAIVE
    # One gradient arena (and one plan over the same weights and state) per step, as far as memory allows, so that
    # every step's fresh gradients are resident before the timed region and the K steps run back to back in it.
    total_steps = args.warmup + args.steps
    free = torch.cuda.mem_get_info()[0]
    base_need = harness.DeviceWorkload.pool_bytes(wl, over.get("mode", eco.ECO_MODE_ECO))
    per_set = 2 * wl.numel + (4 << 20)
    grad_sets = int(max(1, min(total_steps, (0.45 * free - base_need) // per_set + 1)))
    t_setup = time.perf_counter()
    dw = harness.DeviceWorkload(wl, "cuda:0", layout=over, init="bulk" if args.bulk_init else True,
                                placement=args.placement, grad_sets=grad_sets,
                                spread_gap=(args.spread_gap_gib << 30) or None, calibrate_gaps=args.calibrate_gaps)
    fill = dw.fill_gradients_bulk if args.bulk_grad else dw.fill_gradients
    for g in range(grad_sets):
        fill(g + 1, g)                            # step k reads set (k - 1) mod grad_sets
    torch.cuda.synchronize()
    print(f"[bench] {wl.name}: {len(wl.tensors)} tensors, {wl.numel} parameters, {grad_sets} gradient sets, "
          f"placement: {dw.placement}, set-up {time.perf_counter() - t_setup:.1f} s", file=sys.stderr, flush=True)

    k = 0
    for _ in range(args.warmup):
        k += 1
        dw.step(k, (k - 1) % grad_sets)
    torch.cuda.synchronize()

    # the timed region: exactly K steps, nothing else on the device, one synchronize on each side
    events = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    first = k + 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        k += 1
        events[i].record()
        dw.step(k, (k - 1) % grad_sets)
    events[args.steps].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [events[i].elapsed_time(events[i + 1]) for i in range(args.steps)]
    for i, ms in enumerate(kernel_ms):
        print(f"[bench] step {first + i}: {ms:.3f} ms", file=sys.stderr, flush=True)

    ms_per_step = wall / args.steps * 1e3
    value = wl.numel / (ms_per_step * 1e-3)
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) * 1e-3
    alg_bytes = algorithmic_bytes(wl, args.variant)
    achieved = alg_bytes / avg_kernel_s / 1e9
    headline = args.variant == "adam-sr" and args.granularity == "block"
    traffic, traffic_source = profiled_traffic(wl.name) if headline else (None, None)
    out = {
        "metric": METRIC, "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic" if grad_sets >= total_steps else f"synthetic ({grad_sets} gradient sets reused in turn)",
        "config": {"workload": wl.name, "granularity": args.granularity, "tensors": len(wl.tensors), "parameters": wl.numel,
                   "placement": dw.placement,
                   "placement_probe_gib_ms": dw.calibration,
                   "placement_probe": dw.probe_results,
                   "format": ("fp8_e4m3 codes, %s fp32 scales, bf16 gradients, fp32 m and v"
                              if args.config != 5 else "int4 codes, %s bf16 scales, bf16 gradients, bf16 m and v")
                   % {"block": "block-128", "row": "row-wise", "tensor": "tensor-wise"}[args.granularity],
                   "optimizer": args.variant,
                   "static_bytes_per_param": round(static_bytes_per_param(wl, args.variant), 4),
                   "launches_per_step": {"block": 1 if args.config != 2 else 2, "row": "one per row length",
                                         "tensor": "two passes, a reduction and a scale kernel"}[args.granularity]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": avg_kernel_s * 1e3,
                     "kernel_ms_median": sorted(kernel_ms)[len(kernel_ms) // 2], "kernel_ms_min": min(kernel_ms)},
    }
    quantized_only = all(t.fmt in ("fp8", "int4") for t in wl.tensors)
    if not args.no_parity and not args.no_cpu_baseline:
        out["parity"] = parity_step(dw, wl, k + 1, k % grad_sets)
        print(f"[bench] parity: {out['parity']}", file=sys.stderr, flush=True)
    if not args.no_ceiling and args.config in (3, 4) and quantized_only and args.granularity == "block":
        # what the memory system gives the step's access pattern without its arithmetic, on the very arrays just stepped
        # (their contents are scrambled by it: nothing reads them afterwards)
        n = min(dw.m.numel(), dw.codes.numel()) // 1024 * 1024
        mix = time_launches(lambda: eco.eco_bandwidth_probe(0, dw.codes, dw.scales, dw.grad, dw.m, dw.v, n), 5)
        cpy = time_launches(lambda: eco.eco_bandwidth_probe(1, None, None, None, dw.m, dw.v, n), 5)
        out["roofline"]["ceiling_gbs"] = n * 20.0625 / (mix[0] * 1e-3) / 1e9
        out["roofline"]["plain_copy_gbs"] = n * 8.0 / (cpy[0] * 1e-3) / 1e9
        out["roofline"]["ceiling_what"] = ("eco_bandwidth_probe on the same arrays: ceiling_gbs = the step's loads and stores "
                                           "(11.03 B read, 9.03 B written per element, same tiles and occupancy cap) without "
                                           "arithmetic; plain_copy_gbs = float4 copy m -> v; averages of 5 launches")
    placement_used = dw.placement
    dw.close()
    del dw
    torch.cuda.empty_cache()
    if args.compare_placements is None:
        args.compare_placements = "dense,packed,spread" if headline else ""
    others = [p for p in args.compare_placements.split(",") if p] if args.config == 4 else []
    for other in others:
        bulk_ok = over.get("mode", eco.ECO_MODE_ECO) in (eco.ECO_MODE_ECO, eco.ECO_MODE_NAIVE)
        dw2 = harness.DeviceWorkload(wl, "cuda:0", layout=over, init="bulk" if bulk_ok else True, placement=other,
                                     grad_sets=min(grad_sets, 4), calibrate_gaps=0)
        if dw2.placement == placement_used:
            dw2.close()
            continue
        for g in range(len(dw2.grads)):
            dw2.fill_gradients_bulk(g + 1, g)
        torch.cuda.synchronize()
        kk = [0]

        def one():
            kk[0] += 1
            dw2.step(kk[0], (kk[0] - 1) % len(dw2.grads))
        avg, med, mn = time_launches(one, args.steps, warm=args.warmup)
        out.setdefault("other_placements", []).append(
            {"placement": dw2.placement, "kernel_ms": avg, "kernel_ms_median": med, "kernel_ms_min": mn,
             "frac": alg_bytes / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "what": f"the same step, {args.warmup} warm-up + {args.steps} timed launches, arbitrary valid weights"})
        print(f"[bench] placement {dw2.placement}: {avg:.3f} ms", file=sys.stderr, flush=True)
        dw2.close()
        del dw2
        torch.cuda.empty_cache()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
