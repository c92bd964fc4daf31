"""Device-side set-up of a synthetic workload for the ECO library: memory, initial quantization, plan.

PyTorch is used for device memory, streams and random gradients only; every operation of the
method (initial quantization included) is a call into libeco.so through the binding.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import torch

import workloads
from workloads import Workload

from . import binding as eco

_FMT = {"fp8": eco.ECO_FMT_FP8_E4M3, "int4": eco.ECO_FMT_INT4, "bf16_plain": eco.ECO_FMT_BF16_PLAIN,
        "fp32_identity": eco.ECO_FMT_FP32_IDENTITY}


def _round_up(x: int, k: int) -> int:
    return (x + k - 1) // k * k


@dataclass
class TensorViews:
    spec: workloads.TensorSpec
    tensor_id: int
    fmt: int
    weights: torch.Tensor          # uint8 codes, or bf16 / fp32 weights
    scales: Optional[torch.Tensor]
    grad: torch.Tensor             # bf16
    m: torch.Tensor
    v: torch.Tensor
    aux: Optional[torch.Tensor] = None   # fp32 master weights or stored error, when the mode uses one


class DeviceWorkload:
    """All tensors of a workload resident in HBM, carved out of a few flat arenas (one per array
    kind) so that a multi-thousand-tensor model costs a handful of allocations; each tensor still
    has its own descriptor in the plan and its own, 256-byte aligned, slices."""

    # Where the arrays lie in device memory matters on MI355X: measured with the arrays placed by hand inside one
    # 244 GiB allocation, the address space falls into 32 GiB regions of three kinds, and the step (nine streams
    # that advance in lock-step) runs 3 % faster, its loads and stores alone 9 % faster, when the m or the v
    # array lies in a region of another kind than the rest; a plain two-stream copy does not care.  Which region
    # is of which kind is a property of the physical addresses an allocation happens to get.  Placements:
    #   "packed"  one allocation per arena, wherever the allocator puts them;
    #   "dense"   one allocation, no byte unused, order m | codes, scales, gradients | v;
    #   "probed"  one allocation, no byte unused; m first, and v after as many of the other arenas (codes and scales,
    #             then the gradient arenas) as the library's bandwidth probe, run on the candidate addresses before
    #             anything is initialised, finds fastest;
    #   "spread"  one allocation with the arena groups SPREAD_GAP bytes apart: the gaps are memory the benchmark
    #             does not use (kept for comparison).
    SPREAD_GAP = 48 << 30
    SPREAD_MIN_BYTES = 8 << 30          # "auto" spreads workloads of at least this footprint

    def __init__(self, wl: Workload, device: str = "cuda:0", base_seed: int = workloads.BASE_SEED,
                 init=True, layout: Optional[dict] = None, skew_bytes: Optional[dict] = None,
                 single_allocation=False, placement: str = "auto", grad_sets: int = 1,
                 spread_gap: Optional[int] = None, calibrate_gaps: int = 0, order: str = "default"):
        """`layout`: hyper-parameter overrides that are fixed for the life of the plan (opt, mode, ...).
        In the master-weight mode the fp32 initial weights are kept as the master copy; in the
        exact-injection mode the aux buffer starts as e_0 = theta_0 - q(theta_0) (Appendix A).
        `placement`: "packed", "dense", "probed" or "spread" (see the class comment); "auto" = probed for large
        workloads the probe's arrays fit (FP8 codes, fp32 state, Adam, with or without master weights), dense for other
        large ones, packed for small ones.  `skew_bytes` / `single_allocation` place arenas by hand (probes).
        `order`: "default" lays the arenas out as codes, scales, gradients, m, v; "state-apart" (one allocation only)
        puts m first and v last with everything else between them, no byte unused.
        `grad_sets`: number of gradient arenas (each with a plan of its own over the same weights and state),
        so that the gradients of several steps can be resident before the steps run back to back.
        `calibrate_gaps`: with the spread placement, time a few steps (on placeholder data, before the weights
        are initialised) for this many candidate gaps, the default and smaller ones in steps of 8 GiB, inside
        the one allocation, and keep the fastest: which distances suit the memory system best differs a little
        from device to device."""
        self.wl = wl
        self.order = order
        self.layout = dict(layout or {})
        self.mode = self.layout.get("mode", eco.ECO_MODE_ECO if self.layout.get("inject", True) else eco.ECO_MODE_NAIVE)
        self.device = torch.device(device)
        self.base_seed = base_seed
        self.state_dtype = torch.bfloat16 if wl.state_bf16 else torch.float32
        self.scale_dtype = torch.bfloat16 if wl.scale_bf16 else torch.float32
        bs = wl.block_size

        offs, soffs, coffs, woffs, off, soff, code_bytes, woff = self._layout(wl)
        dev = self.device
        skew = dict(skew_bytes or {})
        self.placement = "packed"
        self._arena_order = None
        self.probe_results = None
        large = self.pool_bytes(wl, self.mode, grad_sets) >= self.SPREAD_MIN_BYTES and dev.type == "cuda"
        if placement == "auto":
            placement = ("probed" if self._probe_fits() else "dense") if large else "packed"
        if placement == "probed" and not (dev.type == "cuda" and self._probe_fits()):
            placement = "dense"
        if placement == "spread" and not skew and single_allocation is False and dev.type == "cuda":
            need = self.pool_bytes(wl, self.mode, grad_sets)
            ngaps = 3 if self.mode in (eco.ECO_MODE_EXACT, eco.ECO_MODE_MASTER) else 2
            torch.cuda.empty_cache()
            free = torch.cuda.mem_get_info(dev)[0]
            gap = min(spread_gap or self.SPREAD_GAP, max(0, int(0.7 * free) - need) // ngaps) >> 21 << 21
            if gap >= (24 << 30):
                skew = {"m": gap, "v": gap}
                if ngaps == 3:
                    skew["aux"] = gap
                single_allocation = True
                self.placement = f"one allocation, arena groups {gap >> 30} GiB apart"
        probe_order = placement == "probed" and single_allocation is False and not skew
        if placement in ("dense", "dense-default", "probed") and single_allocation is False and not skew:
            single_allocation = True
            if placement != "dense-default":
                self.order = "state-apart"
            self.placement = ("one allocation, no gaps, order: " +
                              ("m | codes, scales, gradients | v" if placement != "dense-default" else "codes, scales, gradients, m, v"))
        pool_buf, pool_pos = None, 0
        external = isinstance(single_allocation, torch.Tensor)
        if external:                                         # a caller-owned uint8 pool; skew["pool"] = where to start in it
            pool_buf = single_allocation
            pool_pos = (-pool_buf.data_ptr()) % (1 << 21) + skew.pop("pool", 0)
        elif single_allocation:
            pool_buf = torch.zeros(self.pool_bytes(wl, self.mode, grad_sets) + sum(skew.values()), dtype=torch.uint8,
                                   device=dev)
            pool_pos = (-pool_buf.data_ptr()) % (1 << 21)
        self._offs = offs

        def build_views(skew, zero):
            """Carve the arenas (separate allocations: the first byte of arena `kind` sits skew[kind] bytes, a
            multiple of 256, into its own allocation; one allocation: arenas follow each other, each starting
            skew[kind] bytes after a 2 MiB boundary) and the per-tensor views into them."""
            pos = [pool_pos]

            def arena(kind, n, dtype):
                k = skew.get(kind, 0)
                assert k % 256 == 0
                es = torch.empty(0, dtype=dtype).element_size()
                if pool_buf is not None:
                    start = pos[0] + k
                    pos[0] = _round_up(start + n * es, 1 << 21)
                    a = pool_buf[start:start + n * es].view(dtype)
                    if zero:
                        a.zero_()
                    return a
                buf = torch.zeros(n + k // es, dtype=dtype, device=dev)
                return buf[k // es:]

            # the arenas, in the order in which they are laid out when they share one allocation
            want = [("codes", max(code_bytes, 1), torch.uint8), ("scales", max(soff, 1), self.scale_dtype),
                    ("plain", max(woff, 1), torch.bfloat16), ("grad", off, torch.bfloat16)]
            want += [(f"grad_extra{k}", off, torch.bfloat16) for k in range(1, grad_sets)]
            want += [("m", off, self.state_dtype), ("v", off, self.state_dtype)]
            if self.mode in (eco.ECO_MODE_EXACT, eco.ECO_MODE_MASTER):
                want.append(("aux", off, torch.float32))
            if self._arena_order is not None:
                want.sort(key=lambda w: self._arena_order.index(w[0]))
            elif self.order == "state-apart":
                # m first, v last: the two largest arrays of the lock-step streams at the two ends of the footprint,
                # everything else (codes, scales, gradients of all resident steps) between them
                want.sort(key=lambda w: {"m": 0, "v": 2, "aux": 3}.get(w[0], 1))
            got = {name: arena("grad_extra" if name.startswith("grad_extra") else name, n, dt) for name, n, dt in want}
            self.codes, self.scales, self.plain = got["codes"], got["scales"], got["plain"]
            self.grads = [got["grad"]] + [got[f"grad_extra{k}"] for k in range(1, grad_sets)]
            self.grad = self.grads[0]
            self.m, self.v, self.aux = got["m"], got["v"], got.get("aux")
            self.tensors = []
            for i, t in enumerate(wl.tensors):
                n = t.numel
                if t.fmt in ("fp8", "int4"):
                    nbytes = n if t.fmt == "fp8" else (n + 1) // 2
                    w = self.codes[coffs[i]:coffs[i] + nbytes]
                    gs = t.group_size(bs)
                    sc = self.scales[soffs[i]:soffs[i] + (n + gs - 1) // gs]
                else:
                    w = self.plain[woffs[i]:woffs[i] + n]
                    sc = None
                o = offs[i]
                self.tensors.append(TensorViews(t, i, _FMT[t.fmt], w, sc, self.grad[o:o + n], self.m[o:o + n],
                                                self.v[o:o + n], None if self.aux is None else self.aux[o:o + n]))

        self.calibration = None
        if probe_order:
            # Which orders are fast depends on the physical memory the allocation got; one whose candidates all time
            # alike (a v array in another kind of region is worth 9 % to the probe; less than 7 % between the fastest and
            # the slowest candidate is noise) offers no choice: all of it lies in regions of one kind.  Then another allocation is made while
            # this one is still held, so that it gets other memory, up to three in all and only while the device has
            # room; the allocation with the fastest candidate is kept and the others are returned to the device.
            need = pool_buf.numel()
            best = self._probe_orders(pool_buf, pool_pos, off, soff, code_bytes, woff, grad_sets)
            losers, tried = [], 1
            while (best is not None and best["contrast"] < 1.07 and tried < 3 and
                   torch.cuda.mem_get_info(dev)[0] >= need + (8 << 30)):
                try:
                    other_buf = torch.zeros(need, dtype=torch.uint8, device=dev)
                except torch.cuda.OutOfMemoryError:
                    break
                other_pos = (-other_buf.data_ptr()) % (1 << 21)
                other = self._probe_orders(other_buf, other_pos, off, soff, code_bytes, woff, grad_sets)
                tried += 1
                if other["gbs"] > best["gbs"]:
                    losers.append(pool_buf)
                    pool_buf, pool_pos, best = other_buf, other_pos, other
                else:
                    losers.append(other_buf)
                del other_buf
            if losers:
                losers.clear()
                torch.cuda.empty_cache()
            if best is not None:
                self._arena_order, self.probe_results = best["order"], best["results"]
                self.placement = (f"one allocation, no gaps, order chosen at set-up by the library's bandwidth probe among "
                                  f"{best['orders']} orders" + (f" (in the best of {tried} allocations)" if tried > 1 else "") +
                                  f": {best['text']}")
        if calibrate_gaps > 1 and pool_buf is not None and not external and "GiB apart" in self.placement:
            skew = self._calibrate(build_views, pool_buf, skew, calibrate_gaps)
        build_views(skew, zero=external or self.calibration is not None or self.probe_results is not None)
        if init == "bulk":
            self.init_weights_bulk()
        elif init:
            self.init_weights()
        self.plans = [eco.Plan([self.descriptor(tv, g) for tv in self.tensors], self.hparams(1)) for g in range(grad_sets)]
        self.plan = self.plans[0]

    def _probe_fits(self) -> bool:
        """The library's bandwidth probe moves the bytes of the FP8 / fp32-state Adam step; it is run on a workload's own
        arenas where those are at least as large as what it touches: FP8 codes (any scale granularity), fp32 state,
        Adam, with or without master weights."""
        wl = self.wl
        quant = [t for t in wl.tensors if t.fmt in ("fp8", "int4")]
        return (not wl.state_bf16 and len(quant) > 0 and all(t.fmt == "fp8" for t in quant) and
                self.layout.get("opt", eco.ECO_OPT_ADAM) == eco.ECO_OPT_ADAM)

    @staticmethod
    def candidate_orders(fillers: List[List[str]]) -> List[List[str]]:
        """Orders of the arenas the placement probe times.  `fillers`: the arenas other than m and v as units that stay
        together (codes + scales + unquantized weights; each gradient arena; the master weights), in their usual
        order.  m first and v after the first k units, k = 1 .. all; and, mirrored, v last and m before the last k,
        k = 1 .. all but one (k = all is the first family's last order again)."""
        F = len(fillers)
        flat = lambda units: [n for u in units for n in u]
        orders = [["m"] + flat(fillers[:k]) + ["v"] + flat(fillers[k:]) for k in range(1, F + 1)]
        orders += [flat(fillers[:F - k]) + ["m"] + flat(fillers[F - k:]) + ["v"] for k in range(1, F)]
        return orders

    def _probe_orders(self, pool_buf, pool_pos, off, soff, code_bytes, woff, grad_sets):
        """Candidate orders of the arenas, none of which leaves a byte unused: m first and v after the first k of the
        other arenas (codes + scales + unquantized weights as one unit, then the gradient arenas, then the master
        weights if the mode keeps them), k = 1 .. all of them; and, mirrored, v last and m before the last k.  The probe is timed on each candidate's addresses in the
        still uninitialised allocation.  Returns the fastest order with its figures (None if the workload is too small
        to probe); "contrast" = fastest / slowest candidate."""
        scale_bytes = (2 if self.wl.scale_bf16 else 4) * max(soff, 1)
        sizes = {"codes": max(code_bytes, 1), "scales": scale_bytes, "plain": 2 * max(woff, 1), "m": 4 * off, "v": 4 * off}
        grads = ["grad"] + [f"grad_extra{k}" for k in range(1, grad_sets)]
        for g in grads:
            sizes[g] = 2 * off
        fillers = [["codes", "scales", "plain"]] + [[g] for g in grads]
        if self.mode in (eco.ECO_MODE_EXACT, eco.ECO_MODE_MASTER):
            sizes["aux"] = 4 * off
            fillers.append(["aux"])
        numel = min(code_bytes, off) // 1024 * 1024
        if numel == 0:
            return None
        # the probe reads and rewrites one fp32 scale per 128 elements; where the workload's own scale array is smaller
        # (bf16 scales, one scale per row or per tensor) the start of the code array stands in for it
        probe_scales = "scales" if scale_bytes >= numel // 128 * 4 else "codes"
        orders = self.candidate_orders(fillers)
        base = pool_buf.data_ptr()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        results = []
        for idx, order in enumerate(orders):
            at, pos = {}, pool_pos
            for name in order:
                at[name] = pos
                pos = _round_up(pos + sizes[name], 1 << 21)
            assert pos <= pool_buf.numel()
            a = {n: base + at[n] for n in ("codes", "scales", "grad", "m", "v")}
            for i in range(3):                      # one warm-up launch, two timed ones
                eco.eco_bandwidth_probe(0, a["codes"], a[probe_scales], a["grad"], a["m"], a["v"], numel)
                ev[i].record()
            torch.cuda.synchronize(self.device)
            results.append((min(ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])), idx, at))
        best_ms, best, at = min(results)
        gib = lambda x: round((x - pool_pos) / 2**30, 1)
        figures = [{"gib_into_the_allocation": {n: gib(at_[n]) for n in ("m", "v", "codes", "grad")},
                    "probe_gbs": round(numel * 20.0625 / ms / 1e6)} for ms, _, at_ in results]
        units = [{"m": "m", "v": "v", "codes": "codes, scales", "aux": "master weights"}.get(n, "g") for n in orders[best]
                 if n not in ("scales", "plain")]
        runs = []                                                # "g g g" -> "3 gradient arenas"
        for u in units:
            if u == "g" and runs and runs[-1][0] == "g":
                runs[-1][1] += 1
            else:
                runs.append([u, 1])
        text = " | ".join(f"{c} gradient arena{'s' if c > 1 else ''}" if u == "g" else u for u, c in runs)
        return {"order": orders[best], "results": figures, "gbs": numel * 20.0625 / best_ms / 1e6,
                "contrast": max(r[0] for r in results) / best_ms, "orders": len(orders), "text": text}

    def _calibrate(self, build_views, pool_buf, skew, n_candidates):
        """Times the step for the default gap and for smaller ones (steps of 8 GiB, not below 24 GiB) inside
        the allocation already made, on placeholder contents that are valid for every array kind (the byte
        0x3C: E4M3 code 1.5, INT4 nibbles 3 and -4, 0.0115 as bf16 and as fp32), and returns the fastest skews.
        The pool is left dirty: the caller zeroes the arenas it finally carves."""
        gap = skew["m"]
        cands = [g for g in (gap - (8 << 30) * k for k in range(n_candidates)) if g >= (24 << 30)]
        pool_buf.fill_(0x3C)
        results = []
        for g in cands:
            sk = {k: g for k in skew}
            build_views(sk, zero=False)
            plan = eco.Plan([self.descriptor(tv) for tv in self.tensors], self.hparams(1))
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            for k in range(1, 5):                       # two warm-up steps, two timed ones
                plan.step(self.hparams(k))
                if k >= 2:
                    ev[k - 2].record()
            torch.cuda.synchronize(self.device)
            plan.close()
            results.append((ev[0].elapsed_time(ev[2]) / 2.0, g))
        best_ms, best = min(results)
        self.calibration = [(g >> 30, round(ms, 3)) for ms, g in results]
        self.placement = (f"one allocation, arena groups {best >> 30} GiB apart (fastest of "
                          f"{[g >> 30 for g in cands]} GiB in a timing probe at set-up)")
        return {k: best for k in skew}

    @staticmethod
    def _layout(wl: Workload):
        """Offsets of every tensor inside the arenas: element offsets are multiples of 512, which keeps every
        slice (down to 4-bit codes) 256-byte aligned.  Returns (offs, soffs, coffs, woffs) per tensor and the
        arena sizes (elements of m/v/grad, scales, code bytes, elements of unquantized weights)."""
        bs = wl.block_size
        off = soff = code_bytes = woff = 0
        offs, soffs, coffs, woffs = [], [], [], []
        for t in wl.tensors:
            offs.append(off)
            off += _round_up(t.numel, 512)
            if t.fmt in ("fp8", "int4"):
                soffs.append(soff)
                gs = t.group_size(bs)
                soff += _round_up((t.numel + gs - 1) // gs, 128)
                coffs.append(code_bytes)
                nbytes = t.numel if t.fmt == "fp8" else (t.numel + 1) // 2
                code_bytes += _round_up(nbytes, 256)
                woffs.append(-1)
            else:
                soffs.append(-1)
                coffs.append(-1)
                woffs.append(woff)
                woff += _round_up(t.numel, 512)
        return offs, soffs, coffs, woffs, off, soff, code_bytes, woff

    @staticmethod
    def pool_bytes(wl: Workload, mode: int = eco.ECO_MODE_ECO, grad_sets: int = 1) -> int:
        """Bytes one allocation needs to hold every arena of the workload (without skews)."""
        _, _, _, _, off, soff, code_bytes, woff = DeviceWorkload._layout(wl)
        st = 2 if wl.state_bf16 else 4
        sizes = [max(code_bytes, 1), max(soff, 1) * (2 if wl.scale_bf16 else 4), max(woff, 1) * 2, st * off, st * off]
        sizes += [2 * off] * grad_sets
        if mode in (eco.ECO_MODE_EXACT, eco.ECO_MODE_MASTER):
            sizes.append(4 * off)
        return sum(_round_up(x, 1 << 21) + (1 << 21) for x in sizes) + (1 << 21)

    # ------------------------------------------------------------------ set-up
    @property
    def numel(self) -> int:
        return self.wl.numel

    def grad_view(self, tv: TensorViews, gset: int = 0) -> torch.Tensor:
        """The tensor's slice of gradient arena `gset`."""
        if gset == 0:
            return tv.grad
        o = self._offs[tv.tensor_id]
        return self.grads[gset][o:o + tv.spec.numel]

    def descriptor(self, tv: TensorViews, gset: int = 0) -> "eco.eco_tensor_t":
        return eco.make_tensor(tv.weights, tv.scales, self.grad_view(tv, gset), tv.m, tv.v, tv.spec.numel, tv.tensor_id,
                               tv.fmt, aux=tv.aux, group_size=self.group_size(tv))

    def group_size(self, tv: TensorViews) -> int:
        return tv.spec.group_size(self.wl.block_size)

    def hparams(self, step: int, **over) -> "eco.eco_hparams_t":
        wl = self.wl
        kw = dict(block_size=wl.block_size,
                  state_dtype=eco.ECO_DT_BF16 if wl.state_bf16 else eco.ECO_DT_FP32,
                  scale_dtype=eco.ECO_DT_BF16 if wl.scale_bf16 else eco.ECO_DT_FP32,
                  lr=wl.lr_at(step), beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, step=step, seed=self.base_seed)
        kw.update(self.layout)
        kw.update(over)
        return eco.make_hparams(**kw)

    def init_weights(self) -> None:
        """fp32 N(0, sigma) weights -> round-to-nearest quantization by the library."""
        wl = self.wl
        for tv in self.tensors:
            w = workloads.initial_weights(wl, tv.tensor_id, device=self.device, base_seed=self.base_seed)
            if tv.fmt in (eco.ECO_FMT_FP8_E4M3, eco.ECO_FMT_INT4):
                sdt = eco.ECO_DT_BF16 if wl.scale_bf16 else eco.ECO_DT_FP32
                gs = self.group_size(tv)
                eco.eco_quantize_init(w, eco.ECO_DT_FP32, tv.spec.numel, tv.fmt, gs, sdt, tv.weights, tv.scales)
                if self.mode == eco.ECO_MODE_MASTER:
                    tv.aux.copy_(w)
                elif self.mode == eco.ECO_MODE_EXACT:
                    # e_0 = theta_0 - q(theta_0)
                    eco.eco_quantize_error(w, eco.ECO_DT_FP32, tv.weights, tv.scales, tv.spec.numel, tv.fmt, gs, sdt, tv.aux)
            else:
                tv.weights.copy_(w.to(torch.bfloat16))
            del w
        torch.cuda.synchronize(self.device)

    def init_weights_bulk(self) -> None:
        """Valid but arbitrary quantized weights written with a handful of launches over the whole arenas
        (random non-NaN codes, one constant scale; other values than init_weights, same shapes and bytes):
        for runs under a counter-collecting profiler, where every launch is expensive.  Quantized,
        non-master layouts only."""
        assert self.mode in (eco.ECO_MODE_ECO, eco.ECO_MODE_NAIVE)
        g = torch.Generator(device=self.device)
        g.manual_seed(workloads._mix(self.base_seed, 0x77, 0))
        chunk = 1 << 30
        for o in range(0, self.codes.numel(), chunk):
            n = min(chunk, self.codes.numel() - o)
            if all(tv.fmt == eco.ECO_FMT_FP8_E4M3 for tv in self.tensors if tv.scales is not None):
                # magnitude codes 0x00..0x77 (up to 240), random sign bit: never the NaN patterns 0x7F / 0xFF
                x = torch.randint(0, 0x78, (n,), generator=g, device=self.device, dtype=torch.uint8)
                x |= torch.randint(0, 2, (n,), generator=g, device=self.device, dtype=torch.uint8) << 7
            else:
                # two nibbles in [-7, 7]: never the unused code -8
                lo = torch.randint(-7, 8, (n,), generator=g, device=self.device, dtype=torch.int16)
                hi = torch.randint(-7, 8, (n,), generator=g, device=self.device, dtype=torch.int16)
                x = ((lo & 0xF) | ((hi & 0xF) << 4)).to(torch.uint8)
            self.codes[o:o + n].copy_(x)
            del x
        self.scales.fill_(0.02 * 4 / 448 if self.scales.dtype == torch.float32 else 2.0 ** -9)
        torch.cuda.synchronize(self.device)

    def fill_gradients(self, step: int, gset: int = 0) -> None:
        for tv in self.tensors:
            workloads.gradient(self.wl, tv.tensor_id, step, device=self.device, base_seed=self.base_seed,
                               out=self.grad_view(tv, gset))

    def fill_gradients_bulk(self, step: int, gset: int = 0) -> None:
        """Same distribution as fill_gradients, drawn with a handful of generator calls over the whole
        gradient arena instead of one per tensor (other values, far fewer launches): for runs under
        a counter-collecting profiler, where every launch is expensive."""
        wl = self.wl
        grad = self.grads[gset]
        g = torch.Generator(device=self.device)
        g.manual_seed(workloads._mix(self.base_seed, 0x6B, step))
        chunk = 1 << 28
        stds = {tv.spec.grad_std for tv in self.tensors}
        common = stds.pop() if len(stds) == 1 else 1.0
        for o in range(0, grad.numel(), chunk):
            n = min(chunk, grad.numel() - o)
            x = torch.randn(n, generator=g, device=self.device, dtype=torch.float32)
            if common != 1.0:
                x.mul_(common)
            grad[o:o + n].copy_(x)          # fp32 -> bf16: reads 4n bytes, writes 2n bytes
        if stds:
            for tv in self.tensors:
                self.grad_view(tv, gset).mul_(tv.spec.grad_std)
        for tv in self.tensors:
            t = tv.spec
            if t.expert >= 0 and t.expert in workloads.inactive_experts(wl, step, t.layer, self.base_seed):
                self.grad_view(tv, gset).zero_()

    def step(self, step: int, gset: int = 0, **over) -> None:
        (self.plan if gset == 0 else self.plans[gset]).step(self.hparams(step, **over))

    def close(self) -> None:
        self.plan.close()
        for p in self.plans:
            p.close()
