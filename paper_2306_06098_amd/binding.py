"""ctypes binding of libefcp (see include/efcp.h).  Argument marshalling only:
every step of the path runs in the library's HIP kernels.  torch is used for
device memory and streams and nothing else; there is no CPU fallback, and a
missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libefcp.so")

EFCP_OK, EFCP_EINVAL, EFCP_ENOMEM, EFCP_EHIP, EFCP_ENUMERIC = 0, -1, -2, -3, -4
KERNEL_GROUPS = ("ef_hist", "select", "compact", "sp", "coef", "lcg")

VALUES_FP32, VALUES_BF16 = 0, 1

EXPORTS = (
    "efcp_workspace_bytes", "efcp_workspace_bytes_fmt", "efcp_create", "efcp_create_fmt", "efcp_create_ex",
    "efcp_workspace_bytes_ex", "efcp_row_length", "efcp_create_ggt", "efcp_workspace_bytes_ggt", "efcp_step", "efcp_step_ex", "efcp_apply",
    "efcp_apply_noalloc",
    "efcp_destroy", "efcp_get_row",
    "efcp_get_error", "efcp_get_small", "efcp_default_slice_width", "efcp_create_opts", "efcp_workspace_bytes_opts", "efcp_get_geometry", "efcp_state_bytes",
    "efcp_export_state", "efcp_import_state", "efcp_profile_enable",
    "efcp_profile_read", "efcp_last_error",
)

X_GRAD, X_COMPRESSED = 0, 1

_lib = None


class Options(ctypes.Structure):
    """struct efcp_options."""
    _fields_ = [("value_format", ctypes.c_int32), ("topk_block", ctypes.c_int32),
                ("preconditioner", ctypes.c_int32), ("slice_width", ctypes.c_int32),
                ("single_stream", ctypes.c_int32)]


class EfcpError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"libefcp: {what} (status {code})")
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load libefcp.so built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2306_06098_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double
    lib.efcp_workspace_bytes.restype = ctypes.c_size_t
    lib.efcp_workspace_bytes.argtypes = [i64, i32, i64]
    lib.efcp_create.restype = ctypes.c_int
    lib.efcp_create.argtypes = [ctypes.POINTER(vp), i64, i32, i64, dbl, vp, ctypes.c_size_t]
    lib.efcp_workspace_bytes_fmt.restype = ctypes.c_size_t
    lib.efcp_workspace_bytes_fmt.argtypes = [i64, i32, i64, i32]
    lib.efcp_create_fmt.restype = ctypes.c_int
    lib.efcp_create_fmt.argtypes = [ctypes.POINTER(vp), i64, i32, i64, dbl, i32, vp, ctypes.c_size_t]
    lib.efcp_create_ex.restype = ctypes.c_int
    lib.efcp_create_ex.argtypes = [ctypes.POINTER(vp), i64, i32, i64, dbl, i32, i32, vp, ctypes.c_size_t]
    lib.efcp_workspace_bytes_ex.restype = ctypes.c_size_t
    lib.efcp_workspace_bytes_ex.argtypes = [i64, i32, i64, i32, i32]
    lib.efcp_create_ggt.restype = ctypes.c_int
    lib.efcp_create_ggt.argtypes = [ctypes.POINTER(vp), i64, i32, i64, dbl, i32, i32, vp, ctypes.c_size_t]
    lib.efcp_workspace_bytes_ggt.restype = ctypes.c_size_t
    lib.efcp_workspace_bytes_ggt.argtypes = [i64, i32, i64, i32, i32]
    lib.efcp_default_slice_width.restype = i32
    lib.efcp_default_slice_width.argtypes = [i64, i32]
    lib.efcp_row_length.restype = i64
    lib.efcp_row_length.argtypes = [i64, i64, i32]
    lib.efcp_step.restype = ctypes.c_int
    lib.efcp_step.argtypes = [vp, vp, vp, vp]
    lib.efcp_step_ex.restype = ctypes.c_int
    lib.efcp_step_ex.argtypes = [vp, vp, i32, vp, vp, dbl, dbl, vp]
    lib.efcp_apply.restype = ctypes.c_int
    lib.efcp_apply.argtypes = [vp, vp, vp, vp]
    lib.efcp_apply_noalloc.restype = ctypes.c_int
    lib.efcp_apply_noalloc.argtypes = [vp, vp, vp, vp]
    lib.efcp_destroy.restype = ctypes.c_int
    lib.efcp_destroy.argtypes = [vp]
    lib.efcp_get_row.restype = ctypes.c_int
    lib.efcp_get_row.argtypes = [vp, i32, vp, vp]
    lib.efcp_get_error.restype = ctypes.c_int
    lib.efcp_get_error.argtypes = [vp, vp]
    lib.efcp_get_small.restype = ctypes.c_int
    lib.efcp_get_small.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.efcp_create_opts.restype = ctypes.c_int
    lib.efcp_create_opts.argtypes = [ctypes.POINTER(vp), i64, i32, i64, dbl, ctypes.POINTER(Options), vp,
                                     ctypes.c_size_t]
    lib.efcp_workspace_bytes_opts.restype = ctypes.c_size_t
    lib.efcp_workspace_bytes_opts.argtypes = [i64, i32, i64, ctypes.POINTER(Options)]
    lib.efcp_get_geometry.restype = ctypes.c_int
    lib.efcp_get_geometry.argtypes = [vp, vp, vp, vp]
    lib.efcp_state_bytes.restype = ctypes.c_size_t
    lib.efcp_state_bytes.argtypes = [vp]
    lib.efcp_export_state.restype = ctypes.c_int
    lib.efcp_export_state.argtypes = [vp, vp, ctypes.c_size_t]
    lib.efcp_import_state.restype = ctypes.c_int
    lib.efcp_import_state.argtypes = [vp, vp, ctypes.c_size_t]
    lib.efcp_profile_enable.restype = ctypes.c_int
    lib.efcp_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.efcp_profile_read.restype = ctypes.c_int
    lib.efcp_profile_read.argtypes = [vp, vp, vp]
    lib.efcp_last_error.restype = ctypes.c_char_p
    lib.efcp_last_error.argtypes = [vp]
    _lib = lib
    return lib


TOPK_BLOCK = 16384      # EFCP_TOPK_BLOCK


def efcp_workspace_bytes(d: int, m: int, k: int, values: int = VALUES_FP32, topk_block: int = 0,
                         ggt: bool = False, slice_width: int = 0) -> int:
    o = Options(values, topk_block, 1 if ggt else 0, slice_width, 0)
    return int(load_library().efcp_workspace_bytes_opts(d, m, k, ctypes.byref(o)))


class Efcp:
    """One libefcp context: efcp_create / efcp_step / efcp_destroy."""

    def __init__(self, d: int, m: int, k: int, lam: float, workspace=None, values: int = VALUES_FP32,
                 topk_block: int = 0, ggt: bool = False, slice_width: int = 0, single_stream: bool = False):
        """topk_block = 0: global Top-k of k entries; TOPK_BLOCK: Top-k applied in
        blocks of that many coordinates, k entries per block (self.k is then the
        resulting row length, self.k_arg what was passed).  ggt: Sparse GGT
        (EFCP_SPARSE_GGT), `lam` is then its epsilon and m <= 128.  slice_width: coordinates
        per d-slice, 0 = chosen by the library (efcp_options).  single_stream: no internal
        second stream (efcp_options.single_stream)."""
        self._lib = load_library()
        self.d, self.m, self.lam = int(d), int(m), float(lam)
        self.k_arg, self.topk_block = int(k), int(topk_block)
        self.k = int(self._lib.efcp_row_length(self.d, self.k_arg, self.topk_block))
        self.values = int(values)
        self._ctx = ctypes.c_void_p()
        self._workspace = workspace          # torch tensor kept alive, or None
        ws_ptr, ws_bytes = None, 0
        if workspace is not None:
            ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        opts = Options(self.values, self.topk_block, 1 if ggt else 0, int(slice_width), 1 if single_stream else 0)
        rc = self._lib.efcp_create_opts(ctypes.byref(self._ctx), self.d, self.m, self.k_arg, self.lam,
                                        ctypes.byref(opts), ws_ptr, ws_bytes)
        if rc != EFCP_OK:
            self._ctx = ctypes.c_void_p()
            raise EfcpError(rc, "efcp_create failed")

    def _check(self, rc: int):
        if rc != EFCP_OK:
            raise EfcpError(rc, self._lib.efcp_last_error(self._ctx).decode())

    def step_ptr(self, grad_ptr: int, out_ptr: int, stream: int = 0) -> None:
        self._check(self._lib.efcp_step(self._ctx, grad_ptr, out_ptr, stream))

    def step(self, grad, out, stream=None) -> None:
        """grad, out: contiguous float32 CUDA tensors of d elements; out may be
        None (state updated, F^-1 grad not formed).  Runs on `stream` (a
        torch.cuda.Stream) or torch's current stream."""
        import torch
        assert grad.is_cuda and grad.dtype == torch.float32 and grad.is_contiguous() and grad.numel() == self.d
        if out is not None:
            assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == self.d
        s = stream if stream is not None else torch.cuda.current_stream(grad.device)
        self.step_ptr(grad.data_ptr(), out.data_ptr() if out is not None else None, s.cuda_stream)

    def step_ex(self, grad, x_source: int = X_GRAD, out=None, param=None, lr: float = 0.0,
                weight_decay: float = 0.0, stream=None) -> None:
        """efcp_step_ex: x_source X_GRAD / X_COMPRESSED; `out` receives F^-1 x, or
        `param` is updated in place: theta <- (1 - lr*weight_decay)*theta - lr*F^-1 x."""
        import torch
        ok = lambda t: t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == self.d
        assert ok(grad) and (out is None or ok(out)) and (param is None or ok(param))
        s = stream if stream is not None else torch.cuda.current_stream(grad.device)
        self._check(self._lib.efcp_step_ex(self._ctx, grad.data_ptr(), x_source,
                                           out.data_ptr() if out is not None else None,
                                           param.data_ptr() if param is not None else None,
                                           float(lr), float(weight_decay), s.cuda_stream))

    def apply(self, x, out, stream=None) -> None:
        """efcp_apply: out = F^-1 x on the current window; nothing is inserted."""
        import torch
        ok = lambda t: t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == self.d
        assert ok(x) and ok(out)
        s = stream if stream is not None else torch.cuda.current_stream(x.device)
        self._check(self._lib.efcp_apply(self._ctx, x.data_ptr(), out.data_ptr(), s.cuda_stream))

    def apply_noalloc(self, x, out, stream=None) -> None:
        """efcp_apply_noalloc: as apply(), scratch in the library's static device array."""
        import torch
        ok = lambda t: t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == self.d
        assert ok(x) and ok(out)
        s = stream if stream is not None else torch.cuda.current_stream(x.device)
        self._check(self._lib.efcp_apply_noalloc(self._ctx, x.data_ptr(), out.data_ptr(), s.cuda_stream))

    def destroy(self) -> None:
        if getattr(self, "_ctx", None) and self._ctx.value:
            rc = self._lib.efcp_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()
            self._workspace = None
            if rc != EFCP_OK:
                raise EfcpError(rc, "efcp_destroy failed")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- inspection ----
    def get_row(self, slot: int):
        idx = np.empty(self.k, dtype=np.int32)
        val = np.empty(self.k, dtype=np.float32)
        self._check(self._lib.efcp_get_row(self._ctx, slot, idx.ctypes.data, val.ctypes.data))
        return idx, val

    def get_error(self) -> np.ndarray:
        e = np.empty(self.d, dtype=np.float32)
        self._check(self._lib.efcp_get_error(self._ctx, e.ctypes.data))
        return e

    def get_small(self):
        """Returns dict(S, q, coef, tau, step)."""
        S = np.empty((self.m, self.m), dtype=np.float64)
        q = np.empty(self.m, dtype=np.float64)
        coef = np.empty(self.m, dtype=np.float64)
        tau = ctypes.c_uint32()
        step = ctypes.c_int64()
        self._check(self._lib.efcp_get_small(self._ctx, S.ctypes.data, q.ctypes.data, coef.ctypes.data,
                                             ctypes.addressof(tau), ctypes.addressof(step)))
        return dict(S=S, q=q, coef=coef, tau=int(tau.value), step=int(step.value))

    def geometry(self):
        sl, ns, rs = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
        self._check(self._lib.efcp_get_geometry(self._ctx, ctypes.addressof(sl), ctypes.addressof(ns),
                                                ctypes.addressof(rs)))
        return dict(slice=sl.value, n_slices=ns.value, row_stride=rs.value)

    # ---- checkpoint / resume ----
    def export_state(self) -> np.ndarray:
        """The whole state as one uint8 host array."""
        n = int(self._lib.efcp_state_bytes(self._ctx))
        buf = np.empty(n, dtype=np.uint8)
        self._check(self._lib.efcp_export_state(self._ctx, buf.ctypes.data, n))
        return buf

    def import_state(self, buf: np.ndarray) -> None:
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        self._check(self._lib.efcp_import_state(self._ctx, buf.ctypes.data, buf.size))

    # ---- per-kernel timing ----
    def profile_enable(self, on: bool = True) -> None:
        self._check(self._lib.efcp_profile_enable(self._ctx, 1 if on else 0))

    def profile_read(self):
        """Returns (dict kernel group -> total ms, steps covered)."""
        ms = (ctypes.c_double * len(KERNEL_GROUPS))()
        steps = ctypes.c_int64()
        self._check(self._lib.efcp_profile_read(self._ctx, ctypes.addressof(ms), ctypes.addressof(steps)))
        return {n: ms[i] for i, n in enumerate(KERNEL_GROUPS)}, int(steps.value)
