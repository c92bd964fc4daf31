"""Helpers of the GPU parity tests: move tensors between torch (device) and numpy (host), run the
oracle on host copies, and compare element by element.

The comparison bar (stated once, used everywhere):
  * codes, scales and random words: bit-exact, except that at most 1e-6 of the codes may differ
    (stochastic-rounding boundary flips); zero differences are expected, because both sides take
    every decision in identical fp32 arithmetic;
  * m and v: relative difference <= 1e-6 (fp32 state), or equal bfloat16 bit patterns except that at most
    1e-6 of the elements may hold the ADJACENT bfloat16 code (bf16 state).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from oracle import FMT_BF16_PLAIN, FMT_E4M3, FMT_IDENTITY, FMT_INT4, StepConfig

ORACLE_FMT = {0: FMT_E4M3, 1: FMT_INT4, 2: FMT_BF16_PLAIN, 3: FMT_IDENTITY}
MAX_FLIP_RATE = 1e-6
STATE_RTOL = 1e-6


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()


def to_f32(t: torch.Tensor) -> np.ndarray:
    """Host fp32 copy of an fp32 or bf16 tensor (bf16 -> fp32 is exact)."""
    if t.dtype == torch.bfloat16:
        return oracle.bf16_bits_to_f32(bf16_bits(t))
    return t.detach().cpu().numpy().astype(np.float32, copy=True)


def host_copy(tv) -> dict:
    """Host copies of one tensor's arrays (a TensorViews of the harness, or anything shaped like it)."""
    d = dict(grad=bf16_bits(tv.grad), m=to_f32(tv.m), v=to_f32(tv.v) if tv.v is not None else None)
    if getattr(tv, "aux", None) is not None:
        d["aux"] = to_f32(tv.aux)
    if tv.scales is not None:
        d["codes"] = tv.weights.detach().cpu().numpy().copy()
        d["scales"] = to_f32(tv.scales)
    else:
        d["wreal"] = to_f32(tv.weights)
    return d


def oracle_step(o, h: dict, numel: int, cfg: StepConfig) -> None:
    aux = h.get("aux") if cfg.mode in (oracle.MODE_EXACT, oracle.MODE_MASTER) and "codes" in h else None
    rc = o.eco_step(cfg, numel, h["m"], h.get("v"), codes=h.get("codes"), scales=h.get("scales"),
                    wreal=h.get("wreal"), grad_bf16=h["grad"], aux=aux)
    assert rc == 0, rc


def compare(gpu: dict, ref: dict, what: str = "", state_bf16: bool = False) -> dict:
    """Element-wise comparison of two host copies; returns the statistics it asserted on."""
    stats = {}
    n = ref["m"].size
    if "codes" in ref:
        diff = gpu["codes"] != ref["codes"]
        stats["code_mismatch"] = int(diff.sum())
        assert stats["code_mismatch"] <= MAX_FLIP_RATE * n, f"{what}: {stats['code_mismatch']} code bytes differ of {n}"
        sg, sr = gpu["scales"].view(np.uint32), ref["scales"].view(np.uint32)
        stats["scale_mismatch"] = int((sg != sr).sum())
        assert stats["scale_mismatch"] == 0, f"{what}: {stats['scale_mismatch']} scales differ"
    else:
        wg, wr = gpu["wreal"], ref["wreal"]
        stats["weight_mismatch"] = int((wg.view(np.uint32) != wr.view(np.uint32)).sum())
        assert stats["weight_mismatch"] <= MAX_FLIP_RATE * n, f"{what}: {stats['weight_mismatch']} weights differ"
    if "aux" in ref and "aux" in gpu and "codes" in ref:
        stats["aux_bit_mismatch"] = int((gpu["aux"].view(np.uint32) != ref["aux"].view(np.uint32)).sum())
        ok = np.ones(n, bool) if not stats.get("code_mismatch") else ~_elements_of(diff, n)
        a, b = gpu["aux"].astype(np.float64), ref["aux"].astype(np.float64)
        assert np.all(np.abs(a - b)[ok] <= STATE_RTOL * np.maximum(np.abs(b)[ok], 1e-30)), f"{what}: aux differs"
    for key in ("m", "v"):
        if ref.get(key) is None:
            continue
        a, b = gpu[key].astype(np.float64), ref[key].astype(np.float64)
        assert np.all(np.isfinite(a)) and np.all(np.isfinite(b)), f"{what}: non-finite {key}"
        denom = np.maximum(np.abs(b), 1e-30)
        rel = np.abs(a - b) / denom
        stats[f"{key}_max_rel"] = float(rel.max())
        stats[f"{key}_bit_mismatch"] = int((gpu[key].view(np.uint32) != ref[key].view(np.uint32)).sum())
        if state_bf16:
            # distance in bfloat16 codes (sign-magnitude order): 0 expected, 1 tolerated on a 1e-6 fraction
            ga, gb = gpu[key].view(np.uint32) >> 16, ref[key].view(np.uint32) >> 16
            assert not np.any((gpu[key].view(np.uint32) | ref[key].view(np.uint32)) & 0xFFFF), f"{what}: {key} is not bfloat16"
            oa = np.where(ga & 0x8000, -(ga & 0x7FFF).astype(np.int64), (ga & 0x7FFF).astype(np.int64))
            ob = np.where(gb & 0x8000, -(gb & 0x7FFF).astype(np.int64), (gb & 0x7FFF).astype(np.int64))
            assert np.abs(oa - ob).max() <= 1, f"{what}: {key} differs by more than one bfloat16 code"
            assert stats[f"{key}_bit_mismatch"] <= MAX_FLIP_RATE * n, f"{what}: {key} bf16 mismatches"
        else:
            # a flipped code changes e and therefore m legitimately; exclude those elements (there are none expected)
            ok = np.ones(n, bool)
            if "codes" in ref and stats["code_mismatch"]:
                ok = ~_elements_of(diff, n)
            assert np.all(rel[ok] <= STATE_RTOL), f"{what}: {key} max rel err {rel[ok].max():.3e}"
    return stats


def _elements_of(byte_diff: np.ndarray, n: int) -> np.ndarray:
    if byte_diff.size == n:
        return byte_diff
    return np.repeat(byte_diff, 2)[:n]


def step_config(hp, tensor_id: int, fmt: int, elem_offset: int = 0, group_size: int = 0) -> StepConfig:
    """The oracle's view of the library's hyper-parameter struct (group_size: the tensor's own scale group)."""
    return StepConfig(fmt=ORACLE_FMT[fmt], opt=hp.opt, round=hp.round, mode=hp.mode,
                      block_size=group_size or hp.block_size, state_bf16=bool(hp.state_dtype), scale_bf16=bool(hp.scale_dtype),
                      lr=hp.lr, beta1=hp.beta1, beta2=hp.beta2, eps=hp.eps, weight_decay=hp.weight_decay,
                      step=hp.step, seed=hp.seed, elem_offset=elem_offset, tensor_id=tensor_id)
