"""CPU oracle for the BiQGEMM lookup-table multiply: numpy front end of ``biq_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this package; it is
loaded by the tests, by the smoke check and by the benchmark's ``cpu_baseline`` leg.
It shares no code with the GPU library: the C file is compiled on its own with gcc and
all arithmetic is fp64.

Array conventions (paper notation: m outputs, n inputs, b batch, q bit-planes, mu
LUT-unit, C = ceil(n/mu)):  B int8 [q][m][n] of +1/-1, alpha float32 [q][m],
X float32 [b][n], keys uint16 [q][m][C], packed bitmap uint8 [q][m][stride],
tables float64 [C][2**mu][b], Y float64 [b][m].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "biq_oracle.c")
_LIB = os.path.join(_HERE, "libbiq_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no intrinsics, no OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        L, I, P = ctypes.c_long, ctypes.c_int, ctypes.c_void_p
        lib.biqo_num_chunks.restype = L
        lib.biqo_num_chunks.argtypes = [L, I]
        lib.biqo_row_stride_bytes.restype = L
        lib.biqo_row_stride_bytes.argtypes = [L]
        lib.biqo_packed_bits.restype = L
        lib.biqo_packed_bits.argtypes = [L, L, I]
        lib.biqo_pack_keys.argtypes = [P, L, L, I, I, P]
        lib.biqo_pack_bitmap.argtypes = [P, L, L, I, P]
        lib.biqo_keys_from_bitmap.argtypes = [P, L, L, I, I, P]
        lib.biqo_lut_enum.restype = None
        lib.biqo_lut_enum.argtypes = [P, I, P]
        lib.biqo_lut_dp.restype = L
        lib.biqo_lut_dp.argtypes = [P, I, P]
        lib.biqo_build_lut.argtypes = [P, L, L, I, P]
        lib.biqo_gemm_dense_rows.argtypes = [P, P, P, L, L, I, L, P, L, P]
        lib.biqo_gemm_dense.argtypes = [P, P, P, L, L, I, L, P]
        lib.biqo_gemm_lut.argtypes = [P, P, P, L, L, I, L, I, P]
        lib.biqo_quantize_greedy.argtypes = [P, L, L, I, P, P, P]
        lib.biqo_lstm_cell.argtypes = [P, P, P, P, P, L, L, I, L, P, P]
        _lib = lib
    return _lib


class OracleError(ValueError):
    pass


def _check(rc: int, what: str) -> None:
    if rc != 0:
        reason = {-1: "invalid argument", -2: "B holds a value other than +1/-1", -3: "out of memory"}
        raise OracleError("%s: %s" % (what, reason.get(rc, "error %d" % rc)))


def _arr(a, dtype, ndim=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if ndim is not None and a.ndim != ndim:
        raise OracleError("expected %d dimensions, got %d" % (ndim, a.ndim))
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_chunks(n: int, mu: int) -> int:
    return int(_load().biqo_num_chunks(n, mu))


def row_stride_bytes(n: int) -> int:
    return int(_load().biqo_row_stride_bytes(n))


def packed_bits(m: int, n: int, q: int) -> int:
    return int(_load().biqo_packed_bits(m, n, q))


def pack_keys(B, mu: int) -> np.ndarray:
    """Key matrix K[q][m][C] of LUT-unit mu (Sec. III-B)."""
    B = _arr(B, np.int8, 3)
    q, m, n = B.shape
    keys = np.zeros((q, m, num_chunks(n, mu)), dtype=np.uint16)
    _check(_load().biqo_pack_keys(_ptr(B), m, n, q, mu, _ptr(keys)), "pack_keys")
    return keys


def pack_bitmap(B) -> np.ndarray:
    """Packed sign byte stream [q][m][stride], LSB-first, zero padded."""
    B = _arr(B, np.int8, 3)
    q, m, n = B.shape
    out = np.zeros((q, m, row_stride_bytes(n)), dtype=np.uint8)
    _check(_load().biqo_pack_bitmap(_ptr(B), m, n, q, _ptr(out)), "pack_bitmap")
    return out


def keys_from_bitmap(bitmap, n: int, mu: int) -> np.ndarray:
    bitmap = _arr(bitmap, np.uint8, 3)
    q, m, stride = bitmap.shape
    if stride != row_stride_bytes(n):
        raise OracleError("bitmap stride %d does not match n=%d" % (stride, n))
    keys = np.zeros((q, m, num_chunks(n, mu)), dtype=np.uint16)
    _check(_load().biqo_keys_from_bitmap(_ptr(bitmap), m, n, q, mu, _ptr(keys)), "keys_from_bitmap")
    return keys


def lut_enum(x) -> np.ndarray:
    """One table by its definition M_mu . x; len(x) = mu."""
    x = _arr(x, np.float64, 1)
    table = np.zeros(1 << x.shape[0], dtype=np.float64)
    _load().biqo_lut_enum(_ptr(x), x.shape[0], _ptr(table))
    return table


def lut_dp(x):
    """One table by Algorithm 1; returns (table, number of arithmetic operations)."""
    x = _arr(x, np.float64, 1)
    table = np.zeros(1 << x.shape[0], dtype=np.float64)
    ops = _load().biqo_lut_dp(_ptr(x), x.shape[0], _ptr(table))
    return table, int(ops)


def build_lut(X, mu: int) -> np.ndarray:
    """All tables Q[C][2**mu][b] of X [b][n]."""
    X = _arr(X, np.float32, 2)
    b, n = X.shape
    Q = np.zeros((num_chunks(n, mu), 1 << mu, b), dtype=np.float64)
    _check(_load().biqo_build_lut(_ptr(X), n, b, mu, _ptr(Q)), "build_lut")
    return Q


def gemm_dense(B, alpha, X, rows=None) -> np.ndarray:
    """Eq. 2 with W = sum_i alpha_i B_i reconstructed explicitly. Y [b][m] (or [b][len(rows)])."""
    B = _arr(B, np.int8, 3)
    q, m, n = B.shape
    alpha = _arr(alpha, np.float32, 2)
    X = _arr(X, np.float32, 2)
    if alpha.shape != (q, m) or X.shape[1] != n:
        raise OracleError("shape mismatch")
    b = X.shape[0]
    if rows is None:
        Y = np.zeros((b, m), dtype=np.float64)
        rc = _load().biqo_gemm_dense(_ptr(B), _ptr(alpha), _ptr(X), m, n, q, b, _ptr(Y))
    else:
        rows = _arr(rows, np.int64, 1)
        Y = np.zeros((b, rows.shape[0]), dtype=np.float64)
        rc = _load().biqo_gemm_dense_rows(_ptr(B), _ptr(alpha), _ptr(X), m, n, q, b, _ptr(rows),
                                          rows.shape[0], _ptr(Y))
    _check(rc, "gemm_dense")
    return Y


def gemm_lut(keys, alpha, X, mu: int) -> np.ndarray:
    """Algorithm 2 without tiling on a key matrix [q][m][C]. Y [b][m]."""
    keys = _arr(keys, np.uint16, 3)
    q, m, C = keys.shape
    alpha = _arr(alpha, np.float32, 2)
    X = _arr(X, np.float32, 2)
    b, n = X.shape
    if alpha.shape != (q, m) or C != num_chunks(n, mu):
        raise OracleError("shape mismatch")
    Y = np.zeros((b, m), dtype=np.float64)
    _check(_load().biqo_gemm_lut(_ptr(keys), _ptr(alpha), _ptr(X), m, n, q, b, mu, _ptr(Y)), "gemm_lut")
    return Y


def quantize_greedy(W, q: int, with_residuals: bool = False):
    """Greedy binary-coding quantisation of each row of W (Eq. 1): returns (B int8 [q][m][n],
    alpha float64 [q][m]) and, on request, the residual every plane's signs were taken from."""
    W = _arr(W, np.float32, 2)
    m, n = W.shape
    if q < 1:
        raise OracleError("q must be >= 1")
    B = np.zeros((q, m, n), dtype=np.int8)
    alpha = np.zeros((q, m), dtype=np.float64)
    R = np.zeros((q, m, n), dtype=np.float64) if with_residuals else None
    _check(_load().biqo_quantize_greedy(_ptr(W), m, n, q, _ptr(B), _ptr(alpha),
                                        _ptr(R) if R is not None else None), "quantize_greedy")
    return (B, alpha, R) if with_residuals else (B, alpha)


def lstm_cell(B, alpha, bias, X, C_prev):
    """One LSTM cell step on stacked quantised gate matrices (gates i, f, g, o): B int8 [q][4H][n],
    alpha [q][4H], bias [4H], X [b][n] = [x_t ; h_(t-1)], C_prev [b][H].  Returns (h, c) float64 [b][H]."""
    B = _arr(B, np.int8, 3)
    q, m, n = B.shape
    if m % 4:
        raise OracleError("4H rows expected")
    H = m // 4
    alpha = _arr(alpha, np.float32, 2)
    bias = _arr(bias, np.float32, 1)
    X = _arr(X, np.float32, 2)
    C_prev = _arr(C_prev, np.float32, 2)
    b = X.shape[0]
    if alpha.shape != (q, m) or bias.shape != (m,) or X.shape[1] != n or C_prev.shape != (b, H):
        raise OracleError("shape mismatch")
    h = np.zeros((b, H), dtype=np.float64)
    c = np.zeros((b, H), dtype=np.float64)
    _check(_load().biqo_lstm_cell(_ptr(B), _ptr(alpha), _ptr(bias), _ptr(X), _ptr(C_prev), H, n, q, b,
                                  _ptr(h), _ptr(c)), "lstm_cell")
    return h, c
