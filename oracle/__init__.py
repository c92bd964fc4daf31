"""ctypes front end of the CPU oracle (oracle/eco_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.

The C file is compiled twice, once with REAL=float and once with REAL=double;
``get("f32")`` / ``get("f64")`` return a handle on either build.  The float
build is what the GPU results are compared with (both sides must take each
rounding decision in the same precision); the double build is the one pinned to
closed forms and library routines.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ECO_ORACLE_SOURCE: another C file to build and load instead (the mutation test of the pins plants
# mistakes in copies of the oracle and checks that the pins notice); its libraries go next to it.
_SRC = os.environ.get("ECO_ORACLE_SOURCE") or os.path.join(_HERE, "eco_oracle.c")
_OUT_DIR = os.path.dirname(os.path.abspath(_SRC))

FMT_E4M3, FMT_INT4, FMT_IDENTITY, FMT_ADDNOISE, FMT_BF16_PLAIN = range(5)
OPT_ADAM, OPT_SGDM = 0, 1
ROUND_SR, ROUND_RTN = 0, 1
MODE_NAIVE, MODE_ECO, MODE_EXACT, MODE_MASTER = 0, 1, 2, 3


def lib_path(real: str) -> str:
    return os.path.join(_OUT_DIR, f"liboracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile both builds of the oracle with gcc (plain -O2, no contraction)."""
    for real, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", f"-DREAL={ctype}", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class _Cfg(C.Structure):
    _fields_ = [
        ("fmt", C.c_int32), ("opt", C.c_int32), ("round", C.c_int32), ("mode", C.c_int32),
        ("block_size", C.c_int32), ("state_bf16", C.c_int32), ("scale_bf16", C.c_int32), ("reserved", C.c_int32),
        ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
        ("weight_decay", C.c_double),
        ("step", C.c_uint64), ("seed", C.c_uint64), ("elem_offset", C.c_uint64),
        ("tensor_id", C.c_uint32), ("pad", C.c_uint32),
    ]


@dataclass
class StepConfig:
    """Hyper-parameters H of one step (Alg. 1) plus the quantizer description."""
    fmt: int = FMT_E4M3
    opt: int = OPT_ADAM
    round: int = ROUND_SR
    inject: bool = True          # False = naive master-weight removal
    mode: int = -1               # -1: from `inject`; else MODE_NAIVE / MODE_ECO / MODE_EXACT / MODE_MASTER
    block_size: int = 128
    state_bf16: bool = False
    scale_bf16: bool = False
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    step: int = 1
    seed: int = 0
    elem_offset: int = 0
    tensor_id: int = 0

    def _c(self) -> _Cfg:
        mode = self.mode if self.mode >= 0 else int(self.inject)
        return _Cfg(self.fmt, self.opt, self.round, mode, self.block_size, int(self.state_bf16),
                    int(self.scale_bf16), 0, self.lr, self.beta1, self.beta2, self.eps, self.weight_decay,
                    self.step, self.seed & (2**64 - 1), self.elem_offset, self.tensor_id, 0)


def _ptr(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


class Oracle:
    def __init__(self, real: str):
        assert real in ("f32", "f64")
        build()
        self.real = real
        self.dtype = np.float32 if real == "f32" else np.float64
        self._creal = C.c_float if real == "f32" else C.c_double
        self.lib = C.CDLL(lib_path(real))
        L = self.lib
        L.oracle_sizeof_real.restype = C.c_int
        assert L.oracle_sizeof_real() == np.dtype(self.dtype).itemsize
        L.oracle_num_threads.restype = C.c_int
        L.oracle_bf16_round.restype = self._creal
        L.oracle_bf16_round.argtypes = [self._creal]
        for name in ("oracle_encode", "oracle_quantize_rtn", "oracle_dequantize", "oracle_eco_step"):
            getattr(L, name).restype = C.c_int

    # -- small helpers ------------------------------------------------------
    def _arr(self, a):
        a = np.ascontiguousarray(a, dtype=self.dtype)
        return a

    def num_threads(self) -> int:
        return int(self.lib.oracle_num_threads())

    def set_threads(self, n: int) -> None:
        self.lib.oracle_set_threads(C.c_int(n))

    def philox(self, ctr, key) -> np.ndarray:
        c = np.asarray(ctr, dtype=np.uint32).copy()
        k = np.asarray(key, dtype=np.uint32).copy()
        out = np.zeros(4, dtype=np.uint32)
        self.lib.oracle_philox(_ptr(c, C.c_uint32), _ptr(k, C.c_uint32), _ptr(out, C.c_uint32))
        return out

    def philox_fill(self, seed, step, tensor_id, n_words, first_word=0) -> np.ndarray:
        out = np.zeros(n_words, dtype=np.uint32)
        self.lib.oracle_philox_fill(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tensor_id),
                                    C.c_uint64(first_word), C.c_uint64(n_words), _ptr(out, C.c_uint32))
        return out

    def random16(self, seed, step, tensor_id, n, first_elem=0) -> np.ndarray:
        out = np.zeros(n, dtype=np.uint16)
        self.lib.oracle_random16(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(tensor_id),
                                 C.c_uint64(first_elem), C.c_uint64(n), _ptr(out, C.c_uint16))
        return out

    def decode_table(self, fmt) -> np.ndarray:
        out = np.zeros(256 if fmt == FMT_E4M3 else 16, dtype=self.dtype)
        self.lib.oracle_decode_table(C.c_int(fmt), _ptr(out, self._creal))
        return out

    def encode(self, fmt, rnd, y, r16=None) -> np.ndarray:
        y = self._arr(y)
        out = np.zeros(y.size, dtype=np.uint8)
        r = None if r16 is None else np.ascontiguousarray(r16, dtype=np.uint16)
        rc = self.lib.oracle_encode(C.c_int(fmt), C.c_int(rnd), C.c_uint64(y.size), _ptr(y, self._creal),
                                    _ptr(r, C.c_uint16), _ptr(out, C.c_uint8))
        assert rc == 0
        return out

    def bf16_round(self, x: float) -> float:
        return float(self.lib.oracle_bf16_round(self._creal(x)))

    @staticmethod
    def code_bytes(fmt, numel) -> int:
        return numel if fmt == FMT_E4M3 else (numel + 1) // 2

    def quantize_rtn(self, fmt, x, block_size=128, scale_bf16=False):
        x = self._arr(x).ravel()
        nb = (x.size + block_size - 1) // block_size
        codes = np.zeros(self.code_bytes(fmt, x.size), dtype=np.uint8)
        scales = np.zeros(nb, dtype=self.dtype)
        rc = self.lib.oracle_quantize_rtn(C.c_int(fmt), C.c_int(block_size), C.c_int(int(scale_bf16)),
                                          C.c_uint64(x.size), _ptr(x, self._creal), _ptr(codes, C.c_uint8),
                                          _ptr(scales, self._creal))
        assert rc == 0
        return codes, scales

    def dequantize(self, fmt, codes, scales, numel, block_size=128) -> np.ndarray:
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        scales = self._arr(scales)
        out = np.zeros(numel, dtype=self.dtype)
        rc = self.lib.oracle_dequantize(C.c_int(fmt), C.c_int(block_size), C.c_uint64(numel),
                                        _ptr(codes, C.c_uint8), _ptr(scales, self._creal), _ptr(out, self._creal))
        assert rc == 0
        return out

    def eco_step(self, cfg: StepConfig, numel, m, v=None, *, codes=None, scales=None, wreal=None,
                 grad_bf16=None, grad_real=None, xi=None, aux=None, dbg_theta=None, dbg_err=None) -> int:
        """In-place step; every array must be C-contiguous and of this build's dtype
        (codes uint8, grad_bf16 uint16).  Returns the oracle's status (0 = ok)."""
        def chk(a, dt):
            if a is not None:
                assert a.flags["C_CONTIGUOUS"] and a.dtype == dt, (a.dtype, dt)
        for a in (scales, wreal, grad_real, m, v, xi, aux, dbg_theta, dbg_err):
            chk(a, self.dtype)
        chk(codes, np.uint8)
        chk(grad_bf16, np.uint16)
        c = cfg._c()
        R = self._creal
        return int(self.lib.oracle_eco_step(
            C.byref(c), C.c_uint64(numel), _ptr(codes, C.c_uint8), _ptr(scales, R), _ptr(wreal, R),
            _ptr(grad_bf16, C.c_uint16), _ptr(grad_real, R), _ptr(m, R), _ptr(v, R), _ptr(xi, R), _ptr(aux, R),
            _ptr(dbg_theta, R), _ptr(dbg_err, R)))


_cache: dict = {}


def get(real: str = "f32") -> Oracle:
    if real not in _cache:
        _cache[real] = Oracle(real)
    return _cache[real]


# bfloat16 <-> float32 bit reinterpretation (no arithmetic: a bf16 is the top half of an fp32)
def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits_exact(x: np.ndarray) -> np.ndarray:
    """For values already representable in bfloat16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "value is not a bfloat16"
    return (u >> 16).astype(np.uint16)
