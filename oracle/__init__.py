"""ctypes front end of the CPU oracle (oracle/btc_oracle.cpp).

TEST INFRASTRUCTURE, NOT PRODUCT: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package.  It imports nothing from
the HIP package and the HIP package imports nothing from here.

Every function below only marshals numpy arrays into the C++ routines; the
arithmetic is all in btc_oracle.cpp.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "btc_oracle.cpp")
_LIB = os.path.join(_HERE, "libbtc_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no HIP involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c_long, c_int, c_vp = ctypes.c_long, ctypes.c_int, ctypes.c_void_p
        L.btc_oracle_index_bits.restype = c_int
        L.btc_oracle_index_bits.argtypes = [c_int]
        L.btc_oracle_num_chunks.restype = c_long
        L.btc_oracle_num_chunks.argtypes = [c_long, c_int]
        L.btc_oracle_words_per_row.restype = c_long
        L.btc_oracle_words_per_row.argtypes = [c_long, c_int, c_int]
        L.btc_oracle_storage_bits.restype = c_long
        L.btc_oracle_storage_bits.argtypes = [c_long, c_long, c_int, c_int]
        L.btc_oracle_pack.restype = c_int
        L.btc_oracle_pack.argtypes = [c_vp, c_long, c_long, c_int, c_vp]
        L.btc_oracle_unpack.restype = None
        L.btc_oracle_unpack.argtypes = [c_vp, c_long, c_long, c_int, c_vp]
        L.btc_oracle_f16_to_f64.restype = ctypes.c_double
        L.btc_oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
        L.btc_oracle_bf16_to_f64.restype = ctypes.c_double
        L.btc_oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        L.btc_oracle_widen.restype = None
        L.btc_oracle_widen.argtypes = [c_vp, c_long, c_int, c_vp]
        L.btc_oracle_materialise.restype = None
        L.btc_oracle_materialise.argtypes = [c_vp, c_vp, c_vp, c_vp, c_long, c_long, c_int, c_int,
                                             c_vp, c_long, c_vp]
        L.btc_oracle_materialise_groups.restype = None
        L.btc_oracle_materialise_groups.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_long, c_long, c_int, c_int,
                                                    c_vp, c_long, c_vp]
        L.btc_oracle_matmul.restype = None
        L.btc_oracle_matmul.argtypes = [c_vp, c_long, c_long, c_vp, c_long, c_vp]
        L.btc_oracle_transform.restype = None
        L.btc_oracle_transform.argtypes = [c_vp, c_long, c_long, c_long, c_vp, c_vp, c_vp, c_vp]
        L.btc_oracle_quantize_rows.restype = None
        L.btc_oracle_quantize_rows.argtypes = [c_vp, c_long, c_long, c_int, c_vp, c_vp, c_vp]
        L.btc_oracle_assign.restype = None
        L.btc_oracle_assign.argtypes = [c_vp, c_long, c_int, c_vp, c_long, c_vp, c_vp]
        L.btc_oracle_update.restype = c_int
        L.btc_oracle_update.argtypes = [c_vp, c_vp, c_long, c_int, c_vp, c_long]
        _lib = L
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def index_bits(K: int) -> int:
    return lib().btc_oracle_index_bits(int(K))


def num_chunks(n_in: int, v: int) -> int:
    return lib().btc_oracle_num_chunks(int(n_in), int(v))


def words_per_row(n_in: int, v: int, K: int) -> int:
    return lib().btc_oracle_words_per_row(int(n_in), int(v), int(K))


def storage_bits(out: int, n_in: int, v: int, K: int) -> int:
    return lib().btc_oracle_storage_bits(int(out), int(n_in), int(v), int(K))


def pack(idx: np.ndarray, K: int) -> np.ndarray:
    """int32[out][nchunks] -> uint32[out][wpr]; raises on an index outside [0,K)."""
    idx = _c(idx, np.int32)
    out, nchunks = idx.shape
    wpr = (nchunks * index_bits(K) + 31) // 32
    packed = np.empty((out, wpr), dtype=np.uint32)
    rc = lib().btc_oracle_pack(_p(idx), out, nchunks, int(K), _p(packed))
    if rc != 0:
        raise ValueError("index outside [0, K)")
    return packed


def unpack(packed: np.ndarray, nchunks: int, K: int) -> np.ndarray:
    packed = _c(packed, np.uint32)
    out = packed.shape[0]
    assert packed.shape[1] == (nchunks * index_bits(K) + 31) // 32
    idx = np.empty((out, nchunks), dtype=np.int32)
    lib().btc_oracle_unpack(_p(packed), out, int(nchunks), int(K), _p(idx))
    return idx


def f16_to_f64(h: int) -> float:
    return lib().btc_oracle_f16_to_f64(int(h))


def bf16_to_f64(h: int) -> float:
    return lib().btc_oracle_bf16_to_f64(int(h))


def widen(x_bits: np.ndarray, kind: str) -> np.ndarray:
    """uint16 fp16/bf16 bit patterns -> float64 array of the same shape."""
    x_bits = _c(x_bits, np.uint16)
    xd = np.empty(x_bits.shape, dtype=np.float64)
    lib().btc_oracle_widen(_p(x_bits), x_bits.size, {"f16": 0, "bf16": 1}[kind], _p(xd))
    return xd


def materialise(packed, codebook, alpha, mu, n_in: int, v: int, K: int,
                rows: Optional[np.ndarray] = None) -> np.ndarray:
    """W_hat as float64 [nrows][n_in] (all rows, or the listed ones)."""
    packed = _c(packed, np.uint32)
    codebook = _c(codebook, np.uint32)
    alpha = _c(alpha, np.float32)
    mu = _c(mu, np.float32)
    out = packed.shape[0]
    assert packed.shape[1] == words_per_row(n_in, v, K)
    assert alpha.shape == (out,) and mu.shape == (out,)
    # stored indices of a non-power-of-two K may not exceed the table
    assert codebook.shape[0] >= K
    if rows is None:
        nrows, rows_p = out, ctypes.c_void_p(0)
    else:
        rows = _c(rows, np.int64)
        assert rows.min() >= 0 and rows.max() < out
        nrows, rows_p = rows.shape[0], _p(rows)
    W = np.empty((nrows, n_in), dtype=np.float64)
    lib().btc_oracle_materialise(_p(packed), _p(codebook), _p(alpha), _p(mu), out, int(n_in),
                                 int(v), int(K), rows_p, nrows, _p(W))
    return W


def materialise_groups(packed, codebook, alpha, mu, gmap, n_in: int, v: int, K: int,
                       rows: Optional[np.ndarray] = None) -> np.ndarray:
    """W_hat with several (alpha, mu) groups per row: alpha, mu float32 [out][G]; gmap uint32
    [out][ceil(2 n_in / 32)], 2 bits per weight (see btc_oracle.cpp).  float64 [nrows][n_in]."""
    packed = _c(packed, np.uint32)
    codebook = _c(codebook, np.uint32)
    alpha = _c(alpha, np.float32)
    mu = _c(mu, np.float32)
    gmap = _c(gmap, np.uint32)
    out = packed.shape[0]
    G = alpha.shape[1]
    assert alpha.shape == (out, G) and mu.shape == (out, G) and 1 <= G <= 4
    assert packed.shape[1] == words_per_row(n_in, v, K) and gmap.shape == (out, (2 * n_in + 31) // 32)
    assert codebook.shape[0] >= K
    if rows is None:
        nrows, rows_p = out, ctypes.c_void_p(0)
    else:
        rows = _c(rows, np.int64)
        assert rows.min() >= 0 and rows.max() < out
        nrows, rows_p = rows.shape[0], _p(rows)
    W = np.empty((nrows, n_in), dtype=np.float64)
    lib().btc_oracle_materialise_groups(_p(packed), _p(codebook), _p(alpha), _p(mu), _p(gmap), int(G), out, int(n_in),
                                        int(v), int(K), rows_p, nrows, _p(W))
    return W


def linear_groups(packed, codebook, alpha, mu, gmap, x_bits, n_in: int, v: int, K: int, x_kind: str = "f16",
                  rows: Optional[np.ndarray] = None) -> np.ndarray:
    """The layer with several (alpha, mu) groups per row; float64 [M][nrows]."""
    W = materialise_groups(packed, codebook, alpha, mu, gmap, n_in, v, K, rows)
    return matmul(W, widen(np.atleast_2d(x_bits), x_kind))


def matmul(W: np.ndarray, X: np.ndarray) -> np.ndarray:
    """Y[m][r] = sum_k W[r][k] X[m][k]; W float64 [nrows][in], X float64 [M][in]."""
    W = _c(W, np.float64)
    X = _c(X, np.float64)
    nrows, n_in = W.shape
    M = X.shape[0]
    assert X.shape[1] == n_in
    Y = np.empty((M, nrows), dtype=np.float64)
    lib().btc_oracle_matmul(_p(W), nrows, n_in, _p(X), M, _p(Y))
    return Y


def linear(packed, codebook, alpha, mu, x_bits, n_in: int, v: int, K: int,
           x_kind: str = "f16", rows: Optional[np.ndarray] = None) -> np.ndarray:
    """The whole layer: unpack -> materialise W_hat -> multiply.  Serves both
    the decode GEMV (few activation rows) and the prefill GEMM (many); returns
    float64 [M][nrows]."""
    W = materialise(packed, codebook, alpha, mu, n_in, v, K, rows)
    X = widen(np.atleast_2d(x_bits), x_kind)
    return matmul(W, X)


def transform(x_bits, sign_bits, P1, P2, x_kind: str = "f16") -> np.ndarray:
    """The online activation transform X <- X . diag(sigma) . (P1 kron P2); returns float64 [M][n1*n2]."""
    X = widen(np.atleast_2d(x_bits), x_kind)
    P1 = _c(P1, np.float32)
    P2 = _c(P2, np.float32)
    n1, n2 = P1.shape[0], P2.shape[0]
    assert P1.shape == (n1, n1) and P2.shape == (n2, n2) and X.shape[1] == n1 * n2
    sign_bits = _c(sign_bits, np.uint32)
    assert sign_bits.shape == ((n1 * n2 + 31) // 32,)
    Y = np.empty(X.shape, dtype=np.float64)
    lib().btc_oracle_transform(_p(X), X.shape[0], n1, n2, _p(sign_bits), _p(P1), _p(P2), _p(Y))
    return Y


def quantize_rows(x_bits, x_kind: str, bits: int):
    """Min-max quantisation of every activation row to `bits` bits (fp32 arithmetic, see btc_oracle.cpp);
    returns (q int32 [M][n], lo float32 [M], step float32 [M]) with x ~ lo + step * q."""
    X = widen(np.atleast_2d(x_bits), x_kind).astype(np.float32)   # exact: 16-bit values
    M, n = X.shape
    q = np.empty((M, n), dtype=np.int32)
    lo = np.empty(M, dtype=np.float32)
    step = np.empty(M, dtype=np.float32)
    lib().btc_oracle_quantize_rows(_p(X), M, n, int(bits), _p(q), _p(lo), _p(step))
    return q, lo, step


def dequantize_rows(q, lo, step) -> np.ndarray:
    """lo[m] + step[m] * q[m][k] in float64 (the parameters are fp32 numbers, taken exactly)."""
    q = np.asarray(q, dtype=np.float64)
    return np.asarray(lo, dtype=np.float64)[:, None] + np.asarray(step, dtype=np.float64)[:, None] * q


def linear_aq(packed, codebook, alpha, mu, q, lo, step, n_in: int, v: int, K: int,
              rows: Optional[np.ndarray] = None) -> np.ndarray:
    """The layer on quantised activations: dequantise, then the plain product with the materialised
    W_hat; float64 [M][nrows]."""
    W = materialise(packed, codebook, alpha, mu, n_in, v, K, rows)
    return matmul(W, dequantize_rows(q, lo, step))


def assign(vectors, v: int, codebook):
    """E-step: nearest centroid of every v-bit sign pattern; returns (z int32[N], squared distance int32[N])."""
    vectors = _c(vectors, np.uint32)
    codebook = _c(codebook, np.uint32)
    z = np.empty(vectors.shape[0], dtype=np.int32)
    d2 = np.empty(vectors.shape[0], dtype=np.int32)
    lib().btc_oracle_assign(_p(vectors), vectors.shape[0], int(v), _p(codebook), codebook.shape[0], _p(z), _p(d2))
    return z, d2


def update(vectors, z, v: int, codebook) -> np.ndarray:
    """M-step: majority vote per cluster; returns the new codebook (empty clusters keep their centroid)."""
    vectors = _c(vectors, np.uint32)
    z = _c(z, np.int32)
    new = np.array(codebook, dtype=np.uint32, copy=True)
    if lib().btc_oracle_update(_p(vectors), _p(z), vectors.shape[0], int(v), _p(new), new.shape[0]) != 0:
        raise ValueError("assignment outside [0, K)")
    return new
