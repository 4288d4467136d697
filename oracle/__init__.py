"""CPU oracle for the EFCP / Sparse M-FAC step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``efcp_oracle.c`` (plain C, single thread, fp32 for
error feedback / Top-k, fp64 for every scalar product, the coefficient
recursion and the output).  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the GPU library
never does, and this package imports nothing from the GPU package.

Paper passages followed: Algorithm 1 (lines 5-8), the WSM recursion and
eq. (2) of Section "Efficient Full-Matrix Preconditioners", and the sparse
window G=(I,V) of Section "Compressing Preconditioners via Sparsity".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "efcp_oracle.c")
_LIB = os.path.join(_HERE, "libefcp_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "efcp_oracle.h"))):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double
    lib.eo_create.restype = vp
    lib.eo_create.argtypes = [i64, i32, i64, dbl]
    lib.eo_create_fmt.restype = vp
    lib.eo_create_fmt.argtypes = [i64, i32, i64, dbl, ctypes.c_int]
    lib.eo_create_block.restype = vp
    lib.eo_create_block.argtypes = [i64, i32, i64, i64, dbl, ctypes.c_int]
    lib.eo_block_row_length.restype = i64
    lib.eo_block_row_length.argtypes = [i64, i64, i64]
    lib.eo_create_ggt.restype = vp
    lib.eo_create_ggt.argtypes = [i64, i32, i64, dbl, ctypes.c_int, i64]
    lib.eo_jacobi_eigh.restype = ctypes.c_int
    lib.eo_jacobi_eigh.argtypes = [vp, i32, vp, vp]
    lib.eo_bf16_round.restype = ctypes.c_float
    lib.eo_bf16_round.argtypes = [ctypes.c_float]
    lib.eo_destroy.restype = None
    lib.eo_destroy.argtypes = [vp]
    lib.eo_step.restype = ctypes.c_int
    lib.eo_step.argtypes = [vp, vp, vp, vp]
    lib.eo_step_no_output.restype = ctypes.c_int
    lib.eo_step_no_output.argtypes = [vp, vp]
    lib.eo_step_compressed.restype = ctypes.c_int
    lib.eo_step_compressed.argtypes = [vp, vp, vp]
    lib.eo_apply.restype = ctypes.c_int
    lib.eo_apply.argtypes = [vp, vp, vp]
    lib.eo_param_update.restype = None
    lib.eo_param_update.argtypes = [vp, vp, i64, dbl, dbl]
    lib.eo_step_count.restype = i64
    lib.eo_step_count.argtypes = [vp]
    lib.eo_filled.restype = i32
    lib.eo_filled.argtypes = [vp]
    for name in ("eo_error", "eo_gram", "eo_q", "eo_coef"):
        getattr(lib, name).restype = vp
        getattr(lib, name).argtypes = [vp]
    for name in ("eo_row_idx", "eo_row_val"):
        getattr(lib, name).restype = vp
        getattr(lib, name).argtypes = [vp, i32]
    lib.eo_load_row.restype = ctypes.c_int
    lib.eo_load_row.argtypes = [vp, vp, vp]
    lib.eo_topk.restype = ctypes.c_int
    lib.eo_topk.argtypes = [vp, i64, i64, vp, vp]
    lib.eo_coefficients.restype = ctypes.c_int
    lib.eo_coefficients.argtypes = [vp, vp, i32, i32, dbl, vp]
    _lib = lib
    return lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _view(ptr, n, dtype):
    if not ptr:
        return None
    buf = (ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype, count=n)


def topk(a: np.ndarray, k: int):
    """Top-k by magnitude, ties to the lower index.  Returns (idx asc, val)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    if _load().eo_topk(_ptr(a), a.size, k, _ptr(idx), _ptr(val)) != 0:
        raise MemoryError("eo_topk")
    return idx, val


def coefficients(S: np.ndarray, q: np.ndarray, m: int, lam: float) -> np.ndarray:
    """Coefficients of eq. (2) for rows in the order given by S and q."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    n = q.size
    assert S.shape == (n, n)
    coef = np.zeros(n, dtype=np.float64)
    if _load().eo_coefficients(_ptr(S), _ptr(q), n, m, lam, _ptr(coef)) != 0:
        raise MemoryError("eo_coefficients")
    return coef


def jacobi_eigh(A: np.ndarray):
    """Eigenvalues and eigenvectors (columns) of a symmetric matrix, cyclic Jacobi."""
    A = np.array(A, dtype=np.float64, order="C", copy=True)
    n = A.shape[0]
    assert A.shape == (n, n)
    lam = np.empty(n)
    V = np.empty((n, n))
    _load().eo_jacobi_eigh(_ptr(A), n, _ptr(lam), _ptr(V))
    return lam, V


def bf16_round(a: float) -> float:
    """fp32 -> bfloat16 (nearest even) -> fp32, as the oracle stores values."""
    return float(_load().eo_bf16_round(ctypes.c_float(a)))


def param_update(theta: np.ndarray, u: np.ndarray, lr: float, weight_decay: float) -> np.ndarray:
    """theta <- (1 - lr*weight_decay)*theta - lr*u (Algorithm 1 line 9 with
    decoupled weight decay); returns the new fp32 parameters."""
    out = np.array(theta, dtype=np.float32, copy=True)
    u = np.ascontiguousarray(u, dtype=np.float64)
    assert out.size == u.size
    _load().eo_param_update(_ptr(out), _ptr(u), out.size, float(lr), float(weight_decay))
    return out


class Oracle:
    """State of the oracle: error feedback e, window G=(I,V), Gram matrix S."""

    def __init__(self, d: int, m: int, k: int, lam: float, values_bf16: bool = False, block: int = 0,
                 ggt: bool = False):
        """block = 0: global Top-k of k entries.  block = B > 0: Top-k applied in
        blocks of B coordinates, k entries kept per full block; self.k is then
        the resulting row length.  ggt: Sparse GGT instead of Sparse M-FAC, `lam`
        is then its epsilon."""
        self._lib = _load()
        self.d, self.m, self.lam = int(d), int(m), float(lam)
        self.values_bf16 = bool(values_bf16)
        self.block = int(block)
        self.ggt = bool(ggt)
        if self.block:
            self.k_per_block = int(k)
            self.k = int(self._lib.eo_block_row_length(self.d, self.block, self.k_per_block))
        if self.ggt:
            if not self.block:
                self.k = int(k)
            self._st = self._lib.eo_create_ggt(self.d, self.m, int(k), self.lam, int(self.values_bf16),
                                               self.block)
        elif self.block:
            self._st = self._lib.eo_create_block(self.d, self.m, self.block, self.k_per_block, self.lam,
                                                 int(self.values_bf16))
        else:
            self.k = int(k)
            self._st = self._lib.eo_create_fmt(self.d, self.m, self.k, self.lam, int(self.values_bf16))
        if not self._st:
            raise ValueError("eo_create rejected (d, m, k, lambda)")

    def close(self):
        if getattr(self, "_st", None):
            self._lib.eo_destroy(self._st)
            self._st = None

    __del__ = close

    def step(self, g: np.ndarray, x: np.ndarray | None = None) -> np.ndarray:
        """One step; returns y = F^{-1} x (fp64), x = g when not given."""
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.size == self.d
        xp = None
        if x is not None:
            x = np.ascontiguousarray(x, dtype=np.float32)
            assert x.size == self.d
            xp = _ptr(x)
        y = np.empty(self.d, dtype=np.float64)
        if self._lib.eo_step(self._st, _ptr(g), xp, _ptr(y)) != 0:
            raise MemoryError("eo_step")
        return y

    def step_no_output(self, g: np.ndarray) -> None:
        """Error feedback, Top-k and the window update of one step; F^-1 x is not formed."""
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.size == self.d
        if self._lib.eo_step_no_output(self._st, _ptr(g)) != 0:
            raise MemoryError("eo_step_no_output")

    def step_compressed(self, g: np.ndarray) -> np.ndarray:
        """One step that preconditions the compressed accumulator c_t itself."""
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.size == self.d
        y = np.empty(self.d, dtype=np.float64)
        if self._lib.eo_step_compressed(self._st, _ptr(g), _ptr(y)) != 0:
            raise MemoryError("eo_step_compressed")
        return y

    def apply(self, x: np.ndarray) -> np.ndarray:
        """y = F^{-1} x for the current window; no insertion."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.size == self.d
        y = np.empty(self.d, dtype=np.float64)
        if self._lib.eo_apply(self._st, _ptr(x), _ptr(y)) != 0:
            raise MemoryError("eo_apply")
        return y

    def load_row(self, idx: np.ndarray, val: np.ndarray) -> None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        val = np.ascontiguousarray(val, dtype=np.float32)
        assert idx.size == self.k and val.size == self.k
        if self._lib.eo_load_row(self._st, _ptr(idx), _ptr(val)) != 0:
            raise MemoryError("eo_load_row")

    @property
    def t(self) -> int:
        return int(self._lib.eo_step_count(self._st))

    @property
    def filled(self) -> int:
        return int(self._lib.eo_filled(self._st))

    @property
    def newest_slot(self) -> int:
        return (self.t - 1) % self.m

    @property
    def error(self) -> np.ndarray:
        return _view(self._lib.eo_error(self._st), self.d, np.float32)

    def row(self, slot: int):
        i = _view(self._lib.eo_row_idx(self._st, slot), self.k, np.int32)
        v = _view(self._lib.eo_row_val(self._st, slot), self.k, np.float32)
        return i, v

    @property
    def gram(self) -> np.ndarray:
        return _view(self._lib.eo_gram(self._st), self.m * self.m, np.float64).reshape(self.m, self.m)

    @property
    def q(self) -> np.ndarray:
        return _view(self._lib.eo_q(self._st), self.m, np.float64)

    @property
    def coef(self) -> np.ndarray:
        return _view(self._lib.eo_coef(self._st), self.m, np.float64)
