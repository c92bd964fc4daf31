"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP library's harness and the CPU oracle's tests.
It holds NO arithmetic of the method: it only lists tensor shapes and draws
normal weights and bf16 gradients from a seeded torch generator.  Quantizing the
initial weights is the method's business and is done separately by each side.

The five parameter sets stand in for the paper's models (Sec. 4: 30M-800M
transformers, Gemma-3 1B, a sparse-MoE model, DeepSeek-MoE-16B).  The optimizer
step consumes only shapes and gradient values, so seeded tensors of the same
shapes and value distributions replace the C4 / LM1B / OpenAssistant-Guanaco
training runs, none of which is available here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

BASE_SEED = 20260122


@dataclass
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    fmt: str = "fp8"            # "fp8" | "int4" | "bf16_plain"
    grad_std: float = 1e-3
    layer: int = -1             # layer index, -1 for embeddings
    expert: int = -1            # routed-expert index within the layer, -1 if not a routed expert
    granularity: str = "block"  # scale groups: "block" (the workload's block size), "row" (last dimension), "tensor"

    @property
    def numel(self) -> int:
        return int(math.prod(self.shape))

    def group_size(self, block_size: int) -> int:
        """Elements per scale group of this tensor."""
        if self.granularity == "row":
            return int(self.shape[-1])
        if self.granularity == "tensor":
            return self.numel
        return block_size


@dataclass
class Workload:
    name: str
    tensors: List[TensorSpec]
    steps: int
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    state_bf16: bool = False
    scale_bf16: bool = False
    block_size: int = 128
    weight_std: float = 0.02
    n_experts: int = 0           # routed experts per layer (0: dense model)
    n_inactive: int = 0          # routed experts per layer that get all-zero gradients each step
    cosine_lr: bool = False      # lr_k = lr * 0.5 * (1 + cos(pi * (k-1) / steps))

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)

    def lr_at(self, k: int) -> float:
        """Learning rate of step k (1-based); a cosine schedule runs over the workload's `steps` steps and
        starts again after them, so that runs longer than the configuration keep a positive rate."""
        if not self.cosine_lr:
            return self.lr
        return self.lr * 0.5 * (1.0 + math.cos(math.pi * ((k - 1) % self.steps) / self.steps))


def config1() -> Workload:
    return Workload("cfg1_single_1024x1024", [TensorSpec("w", (1024, 1024))], steps=10)


def config2() -> Workload:
    d, f, n_layers, vocab = 512, 2048, 6, 32000
    ts: List[TensorSpec] = []
    for l in range(n_layers):
        ts.append(TensorSpec(f"l{l}.norm1", (d,), "bf16_plain", layer=l))
        for nm in ("q", "k", "v", "o"):
            ts.append(TensorSpec(f"l{l}.{nm}", (d, d), layer=l))
        ts.append(TensorSpec(f"l{l}.norm2", (d,), "bf16_plain", layer=l))
        ts.append(TensorSpec(f"l{l}.up", (f, d), layer=l))
        ts.append(TensorSpec(f"l{l}.down", (d, f), layer=l))
    ts.append(TensorSpec("final_norm", (d,), "bf16_plain"))
    ts.append(TensorSpec("embed", (vocab, d)))
    # gradient scale varied 10x across tensors, geometrically in list order
    n = len(ts)
    for i, t in enumerate(ts):
        t.grad_std = 1e-3 * 10.0 ** (i / (n - 1))
    return Workload("cfg2_30M_transformer", ts, steps=20, lr=3e-4, cosine_lr=True)


def config3() -> Workload:
    d, f, n_layers, vocab = 1152, 6912, 26, 262144
    ts: List[TensorSpec] = []
    for l in range(n_layers):
        ts += [TensorSpec(f"l{l}.q", (1024, d), layer=l), TensorSpec(f"l{l}.k", (256, d), layer=l),
               TensorSpec(f"l{l}.v", (256, d), layer=l), TensorSpec(f"l{l}.o", (d, 1024), layer=l),
               TensorSpec(f"l{l}.gate", (f, d), layer=l), TensorSpec(f"l{l}.up", (f, d), layer=l),
               TensorSpec(f"l{l}.down", (d, f), layer=l)]
    ts.append(TensorSpec("embed", (vocab, d)))
    for t in ts:
        t.grad_std = 5e-4
    return Workload("cfg3_gemma3_1b_shaped", ts, steps=5)


def config4(layers: int = 16, experts: int = 64, vocab: int = 50304) -> Workload:
    """Sparse-MoE-shaped set: the literal shapes of the configuration (gated experts)."""
    d, f = 1024, 1024
    ts: List[TensorSpec] = []
    for l in range(layers):
        for nm in ("q", "k", "v", "o"):
            ts.append(TensorSpec(f"l{l}.{nm}", (d, d), layer=l))
        ts.append(TensorSpec(f"l{l}.router", (experts, d), layer=l))
        for e in range(experts):
            ts += [TensorSpec(f"l{l}.e{e}.gate", (f, d), layer=l, expert=e),
                   TensorSpec(f"l{l}.e{e}.up", (f, d), layer=l, expert=e),
                   TensorSpec(f"l{l}.e{e}.down", (d, f), layer=l, expert=e)]
    ts.append(TensorSpec("embed", (vocab, d)))
    return Workload("cfg4_smoe_2p1b_shaped", ts, steps=5, n_experts=experts, n_inactive=experts // 4)


def config5(layers: int = 28, vocab: int = 102400) -> Workload:
    d, f, routed, shared = 2048, 1408, 64, 2
    ts: List[TensorSpec] = []
    for l in range(layers):
        for nm in ("q", "k", "v", "o"):
            ts.append(TensorSpec(f"l{l}.{nm}", (d, d), "int4", layer=l))
        ts.append(TensorSpec(f"l{l}.router", (routed, d), "int4", layer=l))
        for e in range(routed + shared):
            ex = e if e < routed else -1          # shared experts always receive gradients
            tag = f"e{e}" if e < routed else f"s{e - routed}"
            ts += [TensorSpec(f"l{l}.{tag}.gate", (f, d), "int4", layer=l, expert=ex),
                   TensorSpec(f"l{l}.{tag}.up", (f, d), "int4", layer=l, expert=ex),
                   TensorSpec(f"l{l}.{tag}.down", (d, f), "int4", layer=l, expert=ex)]
    ts.append(TensorSpec("embed", (vocab, d), "int4"))
    for t in ts:
        t.grad_std = 1e-4
    return Workload("cfg5_deepseek_moe_16b_shaped", ts, steps=3, lr=1e-5, state_bf16=True, scale_bf16=True,
                    n_experts=routed, n_inactive=19)


def config6(layers: int = 24, experts: int = 32, vocab: int = 32128) -> Workload:
    """The shapes of the paper's own sparse-MoE model (Sec. 4.2: 2.1 B parameters, 24 layers, hidden 576, intermediate
    2304, 32 experts; only the expert layers are quantized), beside the benchmark's configuration 4, which carries
    the same label with other shapes.  Two-matrix experts (24 x 32 x 2 x 576 x 2304 = 2.04 B: what the stated total
    allows); attention, router and embedding stay bf16.  Rows of 576 and 2304 elements are not whole numbers of
    512-element tiles: with one scale per row (the paper's FP8 granularity, Sec. 4.1) this is the workload that
    shows what bundling rows into workgroups is worth."""
    d, f = 576, 2304
    ts: List[TensorSpec] = []
    for l in range(layers):
        for nm in ("q", "k", "v", "o"):
            ts.append(TensorSpec(f"l{l}.{nm}", (d, d), "bf16_plain", layer=l))
        ts.append(TensorSpec(f"l{l}.router", (experts, d), "bf16_plain", layer=l))
        for e in range(experts):
            ts += [TensorSpec(f"l{l}.e{e}.up", (f, d), layer=l, expert=e),
                   TensorSpec(f"l{l}.e{e}.down", (d, f), layer=l, expert=e)]
    ts.append(TensorSpec("embed", (vocab, d), "bf16_plain"))
    return Workload("cfg6_paper_smoe_2p1b_shapes", ts, steps=5, lr=2e-5, n_experts=experts, n_inactive=experts // 4)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: config6}


def with_granularity(wl: Workload, granularity: str) -> Workload:
    """The same parameter set with the paper's own scale granularities: "row" (row-wise FP8, Sec. 4.1) or
    "tensor" (tensor-wise INT4, Sec. 4.4) on every quantized tensor."""
    for t in wl.tensors:
        if t.fmt in ("fp8", "int4"):
            t.granularity = granularity
    wl.name += "_" + granularity + "wise"
    return wl


def _mix(*xs: int) -> int:
    """Deterministic 63-bit hash of a few integers (splitmix64 finalizer), for generator seeds."""
    h = 0x9E3779B97F4A7C15
    for x in xs:
        h = (h ^ (x & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        h = (h * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 31
        h = (h * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 29
    return h & 0x7FFFFFFFFFFFFFFF


def _gen(device, *xs: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_mix(*xs))
    return g


def initial_weights(wl: Workload, tensor_id: int, device="cpu", base_seed: int = BASE_SEED) -> torch.Tensor:
    """fp32 N(0, weight_std) weights of one tensor, flattened."""
    t = wl.tensors[tensor_id]
    g = _gen(device, base_seed, 0x57, tensor_id)
    w = torch.randn(t.numel, generator=g, device=device, dtype=torch.float32) * wl.weight_std
    if t.fmt == "bf16_plain":            # norm gains start around one
        w += 1.0
    return w


def inactive_experts(wl: Workload, step: int, layer: int, base_seed: int = BASE_SEED) -> set:
    """Routed experts of `layer` whose gradients are all zero at `step`."""
    if wl.n_inactive == 0 or layer < 0:
        return set()
    g = _gen("cpu", base_seed, 0xE0, step, layer)
    perm = torch.randperm(wl.n_experts, generator=g)
    return set(int(x) for x in perm[: wl.n_inactive])


def gradient(wl: Workload, tensor_id: int, step: int, device="cpu", base_seed: int = BASE_SEED,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """bf16 gradient of one tensor at one step (flattened): N(0, grad_std), or zeros for an inactive expert."""
    t = wl.tensors[tensor_id]
    if out is None:
        out = torch.empty(t.numel, device=device, dtype=torch.bfloat16)
    if t.expert >= 0 and t.expert in inactive_experts(wl, step, t.layer, base_seed):
        out.zero_()
        return out
    g = _gen(device, base_seed, 0x6A, step, tensor_id)
    x = torch.randn(t.numel, generator=g, device=device, dtype=torch.float32) * t.grad_std
    out.copy_(x.to(torch.bfloat16))
    return out
