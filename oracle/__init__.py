"""Adam-mini step oracle (CPU, fp64): test infrastructure, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The arithmetic lives in
``adam_mini_oracle.c`` (Algorithm 1 / Algorithm 2 of the paper, executed
literally in double); this file only builds that C file with gcc and marshals
numpy arrays into it.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adam_mini_oracle.c")
_LIB = os.path.join(_HERE, "libadam_mini_oracle.so")

GRAD_F32 = 0
GRAD_BF16 = 1
GRAD_F64 = 2

# statistic of g .* g that feeds v: "mean" is Algorithm 1; the others are the ablation's candidates
REDUCERS = {"mean": 0, "norm1": 1, "norm2": 2, "max": 3, "min": 4}


def compile_c(src: str, out: str) -> str:
    """gcc one C file into a shared library (a second or two)."""
    tmp = out + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", tmp, src, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


def build(force: bool = False) -> str:
    """Compile the C oracle if it is missing or stale; returns the .so path."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    return compile_c(_SRC, _LIB)


class OracleLib:
    """ctypes view of one compiled copy of adam_mini_oracle.c."""

    def __init__(self, path: str):
        lib = ctypes.CDLL(path)
        u64, dbl, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        lib.amo_step_tensor.restype = ctypes.c_int
        lib.amo_step_tensor.argtypes = [vp, vp, vp, vp, ctypes.c_int, u64, u64, ctypes.c_int,
                                        dbl, dbl, dbl, dbl, dbl, u64, ctypes.c_int]
        lib.amo_block_id.restype = u64
        lib.amo_block_id.argtypes = [vp, vp, vp, ctypes.c_uint32, ctypes.c_uint32, u64]
        lib.amo_block_ids_tensor.restype = ctypes.c_int
        lib.amo_block_ids_tensor.argtypes = [vp, vp, vp, ctypes.c_uint32, ctypes.c_uint32, vp]
        lib.amo_num_blocks.restype = u64
        lib.amo_num_blocks.argtypes = [vp, vp, ctypes.c_uint32]
        lib.amo_num_threads.restype = ctypes.c_int
        lib.amo_num_threads.argtypes = []
        self._lib = lib

    def num_threads(self) -> int:
        return int(self._lib.amo_num_threads())

    def set_num_threads(self, n: int) -> None:
        """Host threads the block loop of amo_step_tensor uses from now on (OpenMP runtime call)."""
        f = self._lib.omp_set_num_threads
        f.restype = None
        f.argtypes = [ctypes.c_int]
        f(int(n))

    def step_tensor(self, p: np.ndarray, m: np.ndarray, v: np.ndarray, g: np.ndarray,
                    block_numel: int, hp: "Hyper", t: int, wd_scale: float = 1.0,
                    strided: bool = False, reducer: str = "mean") -> None:
        """One step on one tensor, in place.  p, m: float64[numel]; v:
        float64[numel // block_numel]; g: float32 / float64 / uint16 (bf16 bits).
        The decay coefficient of the tensor is weight_decay * wd_scale.
        strided: the blocks are the columns of the row-major [block_numel, n_blocks] tensor.
        reducer: key of REDUCERS, the block statistic of g .* g ("mean": the method itself)."""
        numel = p.size
        for a in (p, m, v):
            if a.dtype != np.float64 or not a.flags.c_contiguous:
                raise TypeError("oracle state must be contiguous float64")
        if not g.flags.c_contiguous or g.size != numel or m.size != numel:
            raise ValueError("shape mismatch")
        if block_numel <= 0 or numel % block_numel or v.size != numel // block_numel:
            raise ValueError("bad block_numel / v length")
        lam = hp.weight_decay * float(np.float32(wd_scale))
        rc = self._lib.amo_step_tensor(p.ctypes.data, m.ctypes.data, v.ctypes.data,
                                       g.ctypes.data, _grad_dtype_code(g), numel,
                                       block_numel, 1 if strided else 0, hp.lr, hp.beta1, hp.beta2,
                                       hp.eps, lam, t, REDUCERS[reducer])
        if rc != 0:
            raise ValueError("oracle rejected the arguments (rc=%d)" % rc)

    @staticmethod
    def _strided_arg(strided, n):
        if strided is None:
            return None, None
        a = np.ascontiguousarray([1 if x else 0 for x in strided], dtype=np.int32)
        if a.size != n:
            raise ValueError("strided must have one entry per tensor")
        return a, a.ctypes.data

    def block_id(self, numel: Sequence[int], block_numel: Sequence[int], tensor: int, elem: int,
                 strided: Optional[Sequence[bool]] = None) -> int:
        """v index used by element `elem` of tensor `tensor`."""
        n = np.ascontiguousarray(numel, dtype=np.uint64)
        b = np.ascontiguousarray(block_numel, dtype=np.uint64)
        keep, sp = self._strided_arg(strided, len(n))
        r = self._lib.amo_block_id(n.ctypes.data, b.ctypes.data, sp, len(n), tensor, elem)
        if r == 2 ** 64 - 1:
            raise IndexError("tensor/element out of range")
        return int(r)

    def block_ids_tensor(self, numel: Sequence[int], block_numel: Sequence[int], tensor: int,
                         strided: Optional[Sequence[bool]] = None) -> np.ndarray:
        """v index of every element of tensor `tensor` (uint64 array)."""
        n = np.ascontiguousarray(numel, dtype=np.uint64)
        b = np.ascontiguousarray(block_numel, dtype=np.uint64)
        keep, sp = self._strided_arg(strided, len(n))
        out = np.empty(int(n[tensor]), dtype=np.uint64)
        if self._lib.amo_block_ids_tensor(n.ctypes.data, b.ctypes.data, sp, len(n), tensor, out.ctypes.data) != 0:
            raise IndexError("tensor out of range")
        return out

    def num_blocks(self, numel: Sequence[int], block_numel: Sequence[int]) -> int:
        n = np.ascontiguousarray(numel, dtype=np.uint64)
        b = np.ascontiguousarray(block_numel, dtype=np.uint64)
        return int(self._lib.amo_num_blocks(n.ctypes.data, b.ctypes.data, len(n)))


_default = None


def default_lib() -> OracleLib:
    global _default
    if _default is None:
        _default = OracleLib(build())
    return _default


def num_threads() -> int:
    return default_lib().num_threads()


def set_num_threads(n: int) -> None:
    default_lib().set_num_threads(n)


@dataclass
class Hyper:
    """Hyper-parameters of Algorithm 1; values are widened fp32 numbers when
    the run is compared with the GPU library (which receives fp32)."""
    lr: float
    beta1: float
    beta2: float
    eps: float
    weight_decay: float

    @staticmethod
    def from_f32(lr, beta1, beta2, eps, weight_decay) -> "Hyper":
        f = lambda x: float(np.float32(x))
        return Hyper(f(lr), f(beta1), f(beta2), f(eps), f(weight_decay))


def _grad_dtype_code(g: np.ndarray) -> int:
    if g.dtype == np.float32:
        return GRAD_F32
    if g.dtype == np.uint16:      # bf16 bit patterns
        return GRAD_BF16
    if g.dtype == np.float64:
        return GRAD_F64
    raise TypeError("gradient must be float32, float64 or uint16 (bf16 bits), got %s" % g.dtype)


def step_tensor(p, m, v, g, block_numel, hp, t, wd_scale=1.0, strided=False, reducer="mean") -> None:
    default_lib().step_tensor(p, m, v, g, block_numel, hp, t, wd_scale, strided, reducer)


def block_id(numel, block_numel, tensor, elem, strided=None) -> int:
    return default_lib().block_id(numel, block_numel, tensor, elem, strided)


def num_blocks(numel, block_numel) -> int:
    return default_lib().num_blocks(numel, block_numel)


def block_ids_tensor(numel, block_numel, tensor, strided=None) -> np.ndarray:
    return default_lib().block_ids_tensor(numel, block_numel, tensor, strided)


class OracleState:
    """fp64 optimizer state for a list of tensors, stepped with the C oracle.

    numel / block_numel / wd_scale: one entry per tensor.  params0: initial
    parameter values (any float dtype), widened exactly to double.  m and v
    start at zero (implied by the bias-correction terms of Algorithm 1).
    """

    def __init__(self, numel: Sequence[int], block_numel: Sequence[int],
                 wd_scale: Optional[Sequence[float]], params0: Sequence[np.ndarray],
                 lib: Optional[OracleLib] = None, strided: Optional[Sequence[bool]] = None,
                 reducer: Optional[Sequence[str]] = None, storage: str = "f64"):
        """storage = "f64": the state stays in double between steps (the reference the tolerances are
        stated against).  storage = "f32": p, m and v are rounded to fp32 after every step, as a
        library that stores them in fp32 must; comparing against both tells storage rounding from
        arithmetic error when a parity failure is being diagnosed."""
        if storage not in ("f64", "f32"):
            raise ValueError("storage must be 'f64' or 'f32'")
        self.storage = storage
        self.lib = lib or default_lib()
        self.reducer = ["mean"] * len(numel) if reducer is None else [str(x) for x in reducer]
        self.strided = [False] * len(numel) if strided is None else [bool(x) for x in strided]
        self.numel = [int(x) for x in numel]
        self.block_numel = [int(x) for x in block_numel]
        self.wd_scale = [1.0] * len(self.numel) if wd_scale is None else [float(x) for x in wd_scale]
        self.p: List[np.ndarray] = [np.ascontiguousarray(x, dtype=np.float64).reshape(-1).copy() for x in params0]
        self.m: List[np.ndarray] = [np.zeros(n, dtype=np.float64) for n in self.numel]
        self.v: List[np.ndarray] = [np.zeros(n // b, dtype=np.float64)
                                    for n, b in zip(self.numel, self.block_numel)]
        for n, x in zip(self.numel, self.p):
            if x.size != n:
                raise ValueError("params0 size mismatch")
        self.t = 0

    def step(self, grads: Sequence[np.ndarray], hp: Hyper) -> None:
        self.t += 1
        for k, g in enumerate(grads):
            self.lib.step_tensor(self.p[k], self.m[k], self.v[k], np.ascontiguousarray(g).reshape(-1),
                                 self.block_numel[k], hp, self.t, self.wd_scale[k], self.strided[k],
                                 self.reducer[k])
            if self.storage == "f32":
                with np.errstate(over="ignore"):
                    for a in (self.p[k], self.m[k], self.v[k]):
                        a[:] = a.astype(np.float32).astype(np.float64)

    def v_flat(self) -> np.ndarray:
        return np.concatenate(self.v) if self.v else np.zeros(0)
