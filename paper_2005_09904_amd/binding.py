"""ctypes binding of libbiq.so: same names as include/biq.h, argument marshalling only.

Tensors are torch tensors used purely as device memory; every step of the path runs in the
library's HIP kernels.  There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from .build import LIB_PATH

BIQ_OK, BIQ_EINVAL, BIQ_EUNSUPPORTED, BIQ_EWORKSPACE, BIQ_EHIP = 0, -1, -2, -3, -4

EXPORTS = [
    "biq_status_str", "biq_version", "biq_key_row_stride", "biq_packed_bytes", "biq_num_chunks",
    "biq_lut_bytes", "biq_workspace_bytes", "biq_plan_get", "biq_plan_get_lut", "biq_plan_get_mfma", "biq_plan_check", "biq_plan_workspace_bytes",
    "biq_kernel_name", "biq_pack", "biq_unpack_keys", "biq_build_lut", "biq_query", "biq_gemm",
    "biq_gemm_ex", "biq_quantize", "biq_unpack_keys16", "biq_init", "biq_noalloc_scratch_bytes",
    "biq_gemm_noalloc", "biq_gemm_grouped", "biq_lstm_cell",
]


class BiqPlan(ctypes.Structure):
    """Mirror of biq_plan in include/biq.h."""

    _fields_ = [
        ("kernel", ctypes.c_int), ("threads", ctypes.c_int), ("chunks_per_tile", ctypes.c_int),
        ("batch_tile", ctypes.c_int), ("chunk_splits", ctypes.c_int), ("tiles_per_split", ctypes.c_int),
        ("rows_per_wg", ctypes.c_int), ("row_blocks", ctypes.c_int), ("batch_tiles", ctypes.c_int),
        ("lds_bytes", ctypes.c_int), ("row_mode", ctypes.c_int), ("xcd_skew", ctypes.c_int), ("wave_splits", ctypes.c_int), ("table_fill", ctypes.c_int),
        ("input_terms", ctypes.c_int), ("reserved", ctypes.c_int * 1),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


class BiqProblem(ctypes.Structure):
    """Mirror of biq_problem in include/biq.h."""

    _fields_ = [("K", ctypes.c_void_p), ("alpha", ctypes.c_void_p), ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p),
                ("m", ctypes.c_int), ("n", ctypes.c_int), ("q", ctypes.c_int), ("batch", ctypes.c_int)]


class BiqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, status_str(status), status))


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libbiq.so (built in-tree by paper_2005_09904_amd.build). Raises if it is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            "%s not found: build it first (python -m paper_2005_09904_amd.build); "
            "there is no CPU fallback" % path)
    lib = ctypes.CDLL(path)
    I, P, Z = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    PL = ctypes.POINTER(BiqPlan)
    sig = {
        "biq_status_str": (ctypes.c_char_p, [I]),
        "biq_version": (I, []),
        "biq_key_row_stride": (Z, [I]),
        "biq_packed_bytes": (Z, [I, I, I]),
        "biq_num_chunks": (Z, [I, I]),
        "biq_lut_bytes": (Z, [I, I, I]),
        "biq_workspace_bytes": (Z, [I, I, I, I, I]),
        "biq_plan_get": (I, [I, I, I, I, I, PL]),
        "biq_plan_get_lut": (I, [I, I, I, I, I, PL]),
        "biq_plan_get_mfma": (I, [I, I, I, I, I, I, PL]),
        "biq_plan_check": (I, [I, I, I, I, I, PL]),
        "biq_plan_workspace_bytes": (Z, [PL, I, I]),
        "biq_kernel_name": (ctypes.c_char_p, [I]),
        "biq_pack": (I, [P, P, I, I, I, I, P]),
        "biq_unpack_keys": (I, [P, P, I, I, I, I, P]),
        "biq_unpack_keys16": (I, [P, P, I, I, I, I, P]),
        "biq_build_lut": (I, [P, P, I, I, I, P]),
        "biq_query": (I, [P, P, P, P, I, I, I, I, I, P, Z, P]),
        "biq_gemm": (I, [P, P, P, P, I, I, I, I, I, P, Z, P]),
        "biq_gemm_ex": (I, [P, P, P, P, I, I, I, I, I, PL, P, Z, P]),
        "biq_quantize": (I, [P, P, P, I, I, I, P]),
        "biq_init": (I, []),
        "biq_noalloc_scratch_bytes": (Z, []),
        "biq_gemm_noalloc": (I, [P, P, P, P, I, I, I, I, I, P]),
        "biq_gemm_grouped": (I, [ctypes.POINTER(BiqProblem), I, I, P]),
        "biq_lstm_cell": (I, [P, P, P, P, P, P, P, I, I, I, I, I, P]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().biq_status_str(status).decode()


def _check(status: int, what: str) -> None:
    if status != BIQ_OK:
        raise BiqError(status, what)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream (default: torch's current stream)."""
    import torch

    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


# ---- sizes -----------------------------------------------------------------------------

def biq_key_row_stride(n: int) -> int:
    return load_library().biq_key_row_stride(n)


def biq_packed_bytes(m: int, n: int, q: int) -> int:
    return load_library().biq_packed_bytes(m, n, q)


def biq_num_chunks(n: int, mu: int) -> int:
    return load_library().biq_num_chunks(n, mu)


def biq_lut_bytes(n: int, batch: int, mu: int) -> int:
    return load_library().biq_lut_bytes(n, batch, mu)


def biq_workspace_bytes(m: int, n: int, q: int, batch: int, mu: int) -> int:
    return load_library().biq_workspace_bytes(m, n, q, batch, mu)


def biq_plan_get(m: int, n: int, q: int, batch: int, mu: int) -> BiqPlan:
    plan = BiqPlan()
    _check(load_library().biq_plan_get(m, n, q, batch, mu, ctypes.byref(plan)), "biq_plan_get")
    return plan


def biq_plan_get_lut(m: int, n: int, q: int, batch: int, mu: int) -> BiqPlan:
    plan = BiqPlan()
    _check(load_library().biq_plan_get_lut(m, n, q, batch, mu, ctypes.byref(plan)), "biq_plan_get_lut")
    return plan


def biq_plan_get_mfma(m: int, n: int, q: int, batch: int, mu: int, input_terms: int = 3) -> BiqPlan:
    plan = BiqPlan()
    _check(load_library().biq_plan_get_mfma(m, n, q, batch, mu, input_terms, ctypes.byref(plan)),
           "biq_plan_get_mfma")
    return plan


def biq_plan_check(m: int, n: int, q: int, batch: int, mu: int, plan: BiqPlan) -> BiqPlan:
    _check(load_library().biq_plan_check(m, n, q, batch, mu, ctypes.byref(plan)), "biq_plan_check")
    return plan


def biq_plan_workspace_bytes(plan: BiqPlan, m: int, batch: int) -> int:
    return load_library().biq_plan_workspace_bytes(ctypes.byref(plan), m, batch)


def biq_kernel_name(kernel: int) -> str:
    return load_library().biq_kernel_name(kernel).decode()


# ---- operations (device tensors in, device tensors out) ----------------------------------

def biq_pack(B, K, m: int, n: int, q: int, mu: int, stream=None) -> None:
    _check(load_library().biq_pack(_ptr(B), _ptr(K), m, n, q, mu, _stream(stream)), "biq_pack")


def biq_unpack_keys16(K, keys, m: int, n: int, q: int, mu: int, stream=None) -> None:
    _check(load_library().biq_unpack_keys16(_ptr(K), _ptr(keys), m, n, q, mu, _stream(stream)),
           "biq_unpack_keys16")


def biq_quantize(W, K, alpha, m: int, n: int, q: int, stream=None) -> None:
    _check(load_library().biq_quantize(_ptr(W), _ptr(K), _ptr(alpha), m, n, q, _stream(stream)),
           "biq_quantize")


def biq_unpack_keys(K, keys, m: int, n: int, q: int, mu: int, stream=None) -> None:
    _check(load_library().biq_unpack_keys(_ptr(K), _ptr(keys), m, n, q, mu, _stream(stream)),
           "biq_unpack_keys")


def biq_build_lut(X, LUT, n: int, batch: int, mu: int, stream=None) -> None:
    _check(load_library().biq_build_lut(_ptr(X), _ptr(LUT), n, batch, mu, _stream(stream)),
           "biq_build_lut")


def biq_query(K, alpha, LUT, Y, m: int, n: int, q: int, batch: int, mu: int, workspace=None,
              stream=None) -> None:
    _check(load_library().biq_query(_ptr(K), _ptr(alpha), _ptr(LUT), _ptr(Y), m, n, q, batch, mu,
                                    _ptr(workspace), _nbytes(workspace), _stream(stream)), "biq_query")


def biq_gemm(K, alpha, X, Y, m: int, n: int, q: int, batch: int, mu: int, workspace=None,
             stream=None) -> None:
    _check(load_library().biq_gemm(_ptr(K), _ptr(alpha), _ptr(X), _ptr(Y), m, n, q, batch, mu,
                                   _ptr(workspace), _nbytes(workspace), _stream(stream)), "biq_gemm")


def biq_init() -> None:
    _check(load_library().biq_init(), "biq_init")


def biq_noalloc_scratch_bytes() -> int:
    return load_library().biq_noalloc_scratch_bytes()


def biq_gemm_noalloc(K, alpha, X, Y, m: int, n: int, q: int, batch: int, mu: int, stream=None) -> None:
    _check(load_library().biq_gemm_noalloc(_ptr(K), _ptr(alpha), _ptr(X), _ptr(Y), m, n, q, batch, mu,
                                           _stream(stream)), "biq_gemm_noalloc")


class PreparedGroup:
    """A biq_gemm_grouped call with its descriptor array built once.  problems: list of
    (K, alpha, X, Y, m, n, q, batch); the tensors must stay alive and in place."""

    def __init__(self, problems, mu, stream=None):
        self._keep = problems
        self._array = (BiqProblem * len(problems))()
        for d, (K, alpha, X, Y, m, n, q, batch) in zip(self._array, problems):
            d.K, d.alpha, d.X, d.Y = _ptr(K), _ptr(alpha), _ptr(X), _ptr(Y)
            d.m, d.n, d.q, d.batch = m, n, q, batch
        self._args = (self._array, len(problems), mu, _stream(stream))
        self._fn = load_library().biq_gemm_grouped

    def __call__(self) -> None:
        status = self._fn(*self._args)
        if status != BIQ_OK:
            raise BiqError(status, "biq_gemm_grouped")


def biq_gemm_grouped(problems, mu: int, stream=None) -> None:
    PreparedGroup(problems, mu, stream)()


def biq_lstm_cell(K, alpha, bias, X, C_prev, H_out, C_out, hidden: int, n: int, q: int, batch: int, mu: int,
                  stream=None) -> None:
    _check(load_library().biq_lstm_cell(_ptr(K), _ptr(alpha), _ptr(bias), _ptr(X), _ptr(C_prev), _ptr(H_out),
                                        _ptr(C_out), hidden, n, q, batch, mu, _stream(stream)), "biq_lstm_cell")


class PreparedLstmCell:
    """A biq_lstm_cell call with its arguments marshalled once (see PreparedGemm)."""

    def __init__(self, K, alpha, bias, X, C_prev, H_out, C_out, hidden, n, q, batch, mu, stream=None):
        self._keep = (K, alpha, bias, X, C_prev, H_out, C_out)
        self._fn = load_library().biq_lstm_cell
        self._args = (_ptr(K), _ptr(alpha), _ptr(bias), _ptr(X), _ptr(C_prev), _ptr(H_out), _ptr(C_out), hidden, n, q,
                      batch, mu, _stream(stream))

    def __call__(self) -> None:
        status = self._fn(*self._args)
        if status != BIQ_OK:
            raise BiqError(status, "biq_lstm_cell")


class PreparedGemm:
    """A biq_gemm call with its arguments marshalled once: calling the object only crosses the
    C ABI (no tensor attribute lookups per call).  The tensors must stay alive and in place.
    The stream is the one given here, or torch's current stream at preparation time."""

    def __init__(self, K, alpha, X, Y, m, n, q, batch, mu, workspace=None, stream=None, plan=None):
        lib = load_library()
        self._keep = (K, alpha, X, Y, workspace, plan)
        ws_ptr, ws_bytes, st = _ptr(workspace), _nbytes(workspace), _stream(stream)
        if plan is None:
            self._fn = lib.biq_gemm
            self._args = (_ptr(K), _ptr(alpha), _ptr(X), _ptr(Y), m, n, q, batch, mu, ws_ptr, ws_bytes, st)
        else:
            self._fn = lib.biq_gemm_ex
            self._args = (_ptr(K), _ptr(alpha), _ptr(X), _ptr(Y), m, n, q, batch, mu, ctypes.byref(plan),
                          ws_ptr, ws_bytes, st)

    def __call__(self) -> None:
        status = self._fn(*self._args)
        if status != BIQ_OK:
            raise BiqError(status, "biq_gemm")


def biq_gemm_ex(K, alpha, X, Y, m: int, n: int, q: int, batch: int, mu: int, plan: BiqPlan,
                workspace=None, stream=None) -> None:
    _check(load_library().biq_gemm_ex(_ptr(K), _ptr(alpha), _ptr(X), _ptr(Y), m, n, q, batch, mu,
                                      ctypes.byref(plan), _ptr(workspace), _nbytes(workspace),
                                      _stream(stream)), "biq_gemm_ex")
