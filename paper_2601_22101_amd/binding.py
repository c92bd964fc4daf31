"""Thin ctypes binding of libeco.so (include/eco.h): same names, argument marshalling only.

Every step of the ECO path runs in the library's HIP kernels; PyTorch appears here only as the
owner of device memory (``tensor.data_ptr()``) and of the stream.  If the library has not been
built, importing this module raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Iterable, List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ECO_LIB_PATH") or os.path.join(_HERE, "libeco.so")   # override: a tuning variant

ECO_OK, ECO_EINVAL, ECO_EALIGN, ECO_EUNSUPPORTED, ECO_EHIP, ECO_ENOMEM = 0, -1, -2, -3, -4, -5
ECO_FMT_FP8_E4M3, ECO_FMT_INT4, ECO_FMT_BF16_PLAIN, ECO_FMT_FP32_IDENTITY = 0, 1, 2, 3
ECO_OPT_ADAM, ECO_OPT_SGDM = 0, 1
ECO_ROUND_SR, ECO_ROUND_RTN = 0, 1
ECO_DT_FP32, ECO_DT_BF16 = 0, 1
ECO_MODE_NAIVE, ECO_MODE_ECO, ECO_MODE_EXACT, ECO_MODE_MASTER = 0, 1, 2, 3


class eco_tensor_t(C.Structure):
    _fields_ = [("weights", C.c_void_p), ("scales", C.c_void_p), ("grad", C.c_void_p), ("m", C.c_void_p),
                ("v", C.c_void_p), ("aux", C.c_void_p), ("numel", C.c_uint64), ("group_size", C.c_uint64),
                ("tensor_id", C.c_uint32), ("fmt", C.c_int32)]


class eco_hparams_t(C.Structure):
    _fields_ = [("opt", C.c_int32), ("round", C.c_int32), ("mode", C.c_int32), ("block_size", C.c_uint32),
                ("state_dtype", C.c_int32), ("scale_dtype", C.c_int32),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("step", C.c_uint64), ("seed", C.c_uint64)]


class eco_constants_t(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("b1", "omb1", "b2", "omb2", "rbc2", "c1", "eps", "kappa", "lr", "alpha",
                                         "wd", "inv_lr", "inv_lr_beta")]


class EcoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"eco status {status}: {message}")
        self.status = status


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_22101_amd.build` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32
    lib.eco_plan_create.argtypes = [C.POINTER(eco_tensor_t), C.c_size_t, C.POINTER(eco_hparams_t), C.POINTER(vp)]
    lib.eco_plan_destroy.argtypes = [vp]
    lib.eco_step.argtypes = [vp, C.POINTER(eco_hparams_t), vp]
    lib.eco_step_tensors.argtypes = [C.POINTER(eco_tensor_t), C.c_size_t, C.POINTER(eco_hparams_t), vp]
    lib.eco_step_tensors_noalloc.argtypes = [C.POINTER(eco_tensor_t), C.c_size_t, C.POINTER(eco_hparams_t), vp]
    lib.eco_quantize_init.argtypes = [vp, i32, u64, i32, u64, i32, vp, vp, vp]
    lib.eco_dequantize.argtypes = [vp, vp, u64, i32, u64, i32, vp, vp]
    lib.eco_quantize_error.argtypes = [vp, i32, vp, vp, u64, i32, u64, i32, vp, vp]
    lib.eco_bandwidth_probe.argtypes = [i32, vp, vp, vp, vp, vp, u64, vp]
    lib.eco_arith_selftest.argtypes = [i32, C.c_float, u32, u32, vp, vp]
    lib.eco_philox_fill.argtypes = [u64, u64, u32, u64, u64, vp, vp]
    lib.eco_step_constants.argtypes = [C.POINTER(eco_hparams_t), C.POINTER(eco_constants_t)]
    lib.eco_set_option.argtypes = [i32, C.c_int64]
    for name in ("eco_plan_create", "eco_plan_destroy", "eco_step", "eco_step_tensors", "eco_step_tensors_noalloc", "eco_quantize_init",
                 "eco_dequantize", "eco_quantize_error", "eco_bandwidth_probe", "eco_arith_selftest", "eco_philox_fill", "eco_step_constants", "eco_set_option", "eco_version"):
        getattr(lib, name).restype = C.c_int
    lib.eco_status_string.argtypes = [C.c_int]
    lib.eco_status_string.restype = C.c_char_p
    lib.eco_last_error.restype = C.c_char_p
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != ECO_OK:
        raise EcoError(status, (lib.eco_last_error() or b"").decode())


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor, or an integer address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_tensor(weights, scales, grad, m, v, numel: int, tensor_id: int, fmt: int, aux=None,
                group_size: int = 0) -> eco_tensor_t:
    return eco_tensor_t(_ptr(weights), _ptr(scales), _ptr(grad), _ptr(m), _ptr(v), _ptr(aux), numel, group_size,
                        tensor_id, fmt)


def make_hparams(*, opt=ECO_OPT_ADAM, round=ECO_ROUND_SR, inject=True, mode=None, block_size=128,
                 state_dtype=ECO_DT_FP32, scale_dtype=ECO_DT_FP32, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                 weight_decay=0.0, step=1, seed=0) -> eco_hparams_t:
    """`mode` is an ECO_MODE_* value; when omitted, `inject` chooses between ECO (True) and naive (False)."""
    if mode is None:
        mode = ECO_MODE_ECO if inject else ECO_MODE_NAIVE
    return eco_hparams_t(opt, round, mode, block_size, state_dtype, scale_dtype, lr, beta1, beta2, eps,
                         weight_decay, step, seed & (2 ** 64 - 1))


def eco_version() -> int:
    return lib.eco_version()


def eco_status_string(status: int) -> str:
    return lib.eco_status_string(status).decode()


def eco_last_error() -> str:
    return (lib.eco_last_error() or b"").decode()


def eco_set_option(option: int, value: int) -> None:
    _check(lib.eco_set_option(option, value))


def eco_step_constants(hp: eco_hparams_t) -> eco_constants_t:
    out = eco_constants_t()
    _check(lib.eco_step_constants(C.byref(hp), C.byref(out)))
    return out


def eco_plan_create(tensors: Sequence[eco_tensor_t], layout: eco_hparams_t) -> int:
    arr = (eco_tensor_t * len(tensors))(*tensors)
    plan = C.c_void_p()
    _check(lib.eco_plan_create(arr, len(tensors), C.byref(layout), C.byref(plan)))
    return plan.value


def eco_plan_destroy(plan: Optional[int]) -> None:
    _check(lib.eco_plan_destroy(plan))


def eco_step(plan: int, hp: eco_hparams_t, stream=None) -> None:
    _check(lib.eco_step(plan, C.byref(hp), _stream(stream)))


def eco_step_tensors(tensors: Sequence[eco_tensor_t], hp: eco_hparams_t, stream=None) -> None:
    arr = (eco_tensor_t * len(tensors))(*tensors)
    _check(lib.eco_step_tensors(arr, len(tensors), C.byref(hp), _stream(stream)))


def eco_step_tensors_noalloc(tensors: Sequence[eco_tensor_t], hp: eco_hparams_t, stream=None) -> None:
    arr = (eco_tensor_t * len(tensors))(*tensors)
    _check(lib.eco_step_tensors_noalloc(arr, len(tensors), C.byref(hp), _stream(stream)))


def eco_quantize_init(src, src_dtype: int, numel: int, fmt: int, group_size: int, scale_dtype: int, weights, scales,
                      stream=None) -> None:
    _check(lib.eco_quantize_init(_ptr(src), src_dtype, numel, fmt, group_size, scale_dtype, _ptr(weights),
                                 _ptr(scales), _stream(stream)))


def eco_dequantize(weights, scales, numel: int, fmt: int, group_size: int, scale_dtype: int, dst, stream=None) -> None:
    _check(lib.eco_dequantize(_ptr(weights), _ptr(scales), numel, fmt, group_size, scale_dtype, _ptr(dst),
                              _stream(stream)))


def eco_quantize_error(src, src_dtype: int, weights, scales, numel: int, fmt: int, group_size: int, scale_dtype: int, err,
                       stream=None) -> None:
    _check(lib.eco_quantize_error(_ptr(src), src_dtype, _ptr(weights), _ptr(scales), numel, fmt, group_size, scale_dtype,
                                  _ptr(err), _stream(stream)))


def eco_bandwidth_probe(kind: int, codes, scales, grad, m, v, numel: int, stream=None) -> None:
    _check(lib.eco_bandwidth_probe(kind, _ptr(codes), _ptr(scales), _ptr(grad), _ptr(m), _ptr(v), numel, _stream(stream)))


def eco_arith_selftest(kind: int, numerator: float, bits_lo: int, bits_hi: int, mismatches, stream=None) -> None:
    _check(lib.eco_arith_selftest(kind, numerator, bits_lo, bits_hi, _ptr(mismatches), _stream(stream)))


def eco_philox_fill(seed: int, step: int, tensor_id: int, first_word: int, n_words: int, dst, stream=None) -> None:
    _check(lib.eco_philox_fill(seed & (2 ** 64 - 1), step, tensor_id, first_word, n_words, _ptr(dst), _stream(stream)))


class Plan:
    """RAII wrapper: ``with Plan(tensors, layout) as p: p.step(hp)``."""

    def __init__(self, tensors: Sequence[eco_tensor_t], layout: eco_hparams_t):
        self.handle = eco_plan_create(tensors, layout)

    def step(self, hp: eco_hparams_t, stream=None) -> None:
        eco_step(self.handle, hp, stream)

    def close(self) -> None:
        if self.handle:
            h, self.handle = self.handle, None
            eco_plan_destroy(h)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
