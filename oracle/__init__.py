"""ctypes front-end of the CPU oracle (``maddness_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module,
and this module imports nothing from the product package.

Every function takes and returns NumPy arrays on the host; the arithmetic is
all in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "maddness_oracle.c"), os.path.join(_HERE, "maddness_learn_oracle.c")]
_LIB = os.path.join(_HERE, "libmaddness_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        subprocess.check_call([
            "gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
            "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, *_SRCS, "-lm"])
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_hash_row.restype = C.c_int
        _lib.oracle_scan.restype = C.c_int64
        _lib.oracle_encode_scan.restype = C.c_int64
        _lib.oracle_nmse.restype = C.c_double
        _lib.oracle_bucket_loss.restype = C.c_double
        _lib.oracle_select_idxs.restype = C.c_int32
        _lib.oracle_ridge_prototypes.restype = C.c_int32
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.asarray(a)
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a


def _rows(a):
    """fp32 matrix whose rows may be strided (row stride in elements = strides[0] // 4)."""
    a = np.asarray(a)
    assert a.dtype == np.float32 and a.ndim == 2 and a.strides[1] == 4 and a.strides[0] % 4 == 0
    return a


def hash_row(x, j, v) -> int:
    """Algorithm 1 on one vector; returns the 1-based leaf index."""
    x = _f32(x); v = _f32(v)
    j = np.ascontiguousarray(j, dtype=np.int32)
    assert j.shape == (4,) and v.shape == (16,)
    return int(_L().oracle_hash_row(_p(x), _p(j), _p(v)))


def encode(A, split_dims, thresholds):
    """codes[N][C] in 0..15 (one byte per code, not packed)."""
    A = _rows(A)
    N, _ = A.shape
    split_dims = np.ascontiguousarray(split_dims, dtype=np.int32)
    thresholds = _f32(thresholds)
    Cc = split_dims.shape[0]
    assert split_dims.shape == (Cc, 4) and thresholds.shape == (Cc, 16)
    codes = np.empty((N, Cc), dtype=np.uint8)
    _L().oracle_encode(_p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), C.c_int32(Cc),
                       _p(split_dims), _p(thresholds), _p(codes))
    return codes


DTYPES = {"f32": 0, "f16": 1, "bf16": 2, "u8": 3}
_STORAGE = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16, "u8": np.uint8}


def widen(a, dtype: str):
    """The fp32 numbers with the values of `a` (binary16 given as numpy float16 or as
    its uint16 bit patterns, bfloat16 as uint16 bit patterns, bytes as uint8)."""
    a = np.ascontiguousarray(a)
    if dtype == "f16" and a.dtype == np.uint16:
        a = a.view(np.float16)
    assert a.dtype == _STORAGE[dtype], (a.dtype, dtype)
    out = np.empty(a.shape, dtype=np.float32)
    rc = _L().oracle_widen(_p(a), C.c_int32(DTYPES[dtype]), C.c_int64(a.size), _p(out))
    assert rc == 0
    return out


def encode_typed(A, dtype: str, col_major: bool, split_dims, thresholds):
    """g(A) for A of any supported type; col_major: A is given as the [D][N] array of
    its columns.  Returns codes[N][C] (one byte per code)."""
    A = np.ascontiguousarray(A)
    if dtype == "f16" and A.dtype == np.uint16:
        A = A.view(np.float16)
    assert A.dtype == _STORAGE[dtype] and A.ndim == 2
    N, D = (A.shape[1], A.shape[0]) if col_major else A.shape
    lda = A.shape[1]
    split_dims = np.ascontiguousarray(split_dims, dtype=np.int32)
    thresholds = _f32(thresholds)
    Cc = split_dims.shape[0]
    codes = np.empty((N, Cc), dtype=np.uint8)
    row = np.empty(D, dtype=np.float32)
    rc = _L().oracle_encode_typed(_p(A), C.c_int32(DTYPES[dtype]), C.c_int32(1 if col_major else 0),
                                  C.c_int64(N), C.c_int32(D), C.c_int64(lda), C.c_int32(Cc),
                                  _p(split_dims), _p(thresholds), _p(codes), _p(row))
    assert rc == 0
    return codes


def pack(codes):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, Cc = codes.shape
    out = np.empty((N, (Cc + 1) // 2), dtype=np.uint8)
    _L().oracle_pack(_p(codes), C.c_int64(N), C.c_int32(Cc), _p(out))
    return out


def build_luts_f64(P, B):
    """T[C][16][M] in fp64."""
    P = _f32(P); B = _f32(B)
    Cc, K, D = P.shape
    assert K == 16 and B.shape[0] == D
    M = B.shape[1]
    T = np.empty((Cc, 16, M), dtype=np.float64)
    _L().oracle_build_luts_f64(_p(P), _p(B), C.c_int32(D), C.c_int32(M), C.c_int64(M),
                               C.c_int32(Cc), _p(T))
    return T


def quantize_luts(T):
    """Returns (luts u8 [C][16][M], scale f32 [M], offset f32 [M], l i32 [M], delta f64 [C][M])."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    Cc, K, M = T.shape
    assert K == 16
    luts = np.empty((Cc, 16, M), dtype=np.uint8)
    scale = np.empty(M, dtype=np.float32)
    offset = np.empty(M, dtype=np.float32)
    l = np.empty(M, dtype=np.int32)
    delta = np.empty((Cc, M), dtype=np.float64)
    _L().oracle_quantize_luts(_p(T), C.c_int32(Cc), C.c_int32(M), _p(luts), _p(scale),
                              _p(offset), _p(l), _p(delta))
    return luts, scale, offset, l, delta


def quantize_luts_pooled(T):
    """Appendix A as printed (one scale, one offset per codebook).
    Returns (luts, scale [M], offset [M], l int, delta f64 [C])."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    Cc, K, M = T.shape
    assert K == 16
    luts = np.empty((Cc, 16, M), dtype=np.uint8)
    scale = np.empty(M, dtype=np.float32)
    offset = np.empty(M, dtype=np.float32)
    l = np.empty(1, dtype=np.int32)
    delta = np.empty(Cc, dtype=np.float64)
    _L().oracle_quantize_luts_pooled(_p(T), C.c_int32(Cc), C.c_int32(M), _p(luts), _p(scale),
                                     _p(offset), _p(l), _p(delta))
    return luts, scale, offset, int(l[0]), delta


def scan(packed, Cc, luts, scale, offset, want_acc32=False):
    """Returns (out f32 [N][M], acc16 u16 [N][M], n_overflow[, acc32])."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    luts = np.ascontiguousarray(luts, dtype=np.uint8)
    scale = _f32(scale); offset = _f32(offset)
    N = packed.shape[0]
    assert packed.shape[1] == (Cc + 1) // 2 and luts.shape[:2] == (Cc, 16)
    M = luts.shape[2]
    out = np.empty((N, M), dtype=np.float32)
    acc16 = np.empty((N, M), dtype=np.uint16)
    acc32 = np.empty((N, M), dtype=np.uint32) if want_acc32 else None
    ov = _L().oracle_scan(_p(packed), C.c_int64(N), C.c_int32(Cc), C.c_int32(M), _p(luts),
                          _p(scale), _p(offset), _p(out), C.c_int64(M), _p(acc32), _p(acc16))
    if want_acc32:
        return out, acc16, int(ov), acc32
    return out, acc16, int(ov)


def scan_averaged(packed, Cc, luts, scale, offset, U=16):
    """f by pairwise averages (Appendix D).  Returns (out f32 [N][M], U * sum of block averages u16 [N][M])."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    luts = np.ascontiguousarray(luts, dtype=np.uint8)
    scale = _f32(scale); offset = _f32(offset)
    N = packed.shape[0]
    M = luts.shape[2]
    out = np.empty((N, M), dtype=np.float32)
    usum = np.empty((N, M), dtype=np.uint16)
    rc = _L().oracle_scan_averaged(_p(packed), C.c_int64(N), C.c_int32(Cc), C.c_int32(M), _p(luts),
                                   _p(scale), _p(offset), C.c_int32(U), _p(out), C.c_int64(M), _p(usum))
    if rc != 0:
        raise ValueError("U must be a power of two that divides C")
    return out, usum


def scan_f64(packed, Cc, T):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    T = np.ascontiguousarray(T, dtype=np.float64)
    N = packed.shape[0]
    M = T.shape[2]
    out = np.empty((N, M), dtype=np.float64)
    _L().oracle_scan_f64(_p(packed), C.c_int64(N), C.c_int32(Cc), C.c_int32(M), _p(T), _p(out))
    return out


def encode_scan(A, split_dims, thresholds, luts, scale, offset):
    """Returns (out f32 [N][M], acc16 u16 [N][M], packed codes u8 [N][ceil(C/2)])."""
    A = _rows(A)
    N = A.shape[0]
    split_dims = np.ascontiguousarray(split_dims, dtype=np.int32)
    thresholds = _f32(thresholds)
    luts = np.ascontiguousarray(luts, dtype=np.uint8)
    scale = _f32(scale); offset = _f32(offset)
    Cc = split_dims.shape[0]
    M = luts.shape[2]
    out = np.empty((N, M), dtype=np.float32)
    acc16 = np.empty((N, M), dtype=np.uint16)
    codes = np.empty((N, Cc), dtype=np.uint8)
    packed = np.empty((N, (Cc + 1) // 2), dtype=np.uint8)
    ov = _L().oracle_encode_scan(_p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), C.c_int32(Cc),
                                 _p(split_dims), _p(thresholds), C.c_int32(M), _p(luts),
                                 _p(scale), _p(offset), _p(out), C.c_int64(M), _p(acc16),
                                 _p(codes), _p(packed))
    assert ov == 0, "accumulator exceeds 16 bits"
    return out, acc16, packed


def matmul_f64(A, B):
    A = _rows(A); B = _f32(B)
    N, D = A.shape
    M = B.shape[1]
    Y = np.empty((N, M), dtype=np.float64)
    _L().oracle_matmul_f64(_p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), _p(B),
                           C.c_int32(D), C.c_int32(M), C.c_int64(M), _p(Y))
    return Y


def nmse(Yhat, Y) -> float:
    Yhat = _f32(Yhat)
    Y = np.ascontiguousarray(Y, dtype=np.float64)
    N, M = Y.shape
    return float(_L().oracle_nmse(_p(Yhat), C.c_int64(Yhat.strides[0] // 4), _p(Y),
                                  C.c_int64(N), C.c_int32(M)))


# ----------------------------------------------------------------------------
# learning step (maddness_learn_oracle.c): Section 4.2-4.3, Appendix C
# ----------------------------------------------------------------------------

def _rows_i64(rows):
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1
    return rows


def bucket_loss(X, rows, j) -> float:
    """L(j, B) of Section 4.2 for the bucket `rows` of X and column j."""
    X = _rows(X); rows = _rows_i64(rows)
    return float(_L().oracle_bucket_loss(_p(X), C.c_int64(X.strides[0] // 4), _p(rows), C.c_int64(rows.size),
                                         C.c_int32(j)))


def cumulative_sse(X, reverse: bool):
    """Algorithm 4 on the rows of X (contiguous n x d)."""
    X = _f32(X)
    n, d = X.shape
    out = np.zeros(n, dtype=np.float64)
    _L().oracle_cumulative_sse(_p(X), C.c_int64(n), C.c_int32(d), C.c_int32(1 if reverse else 0), _p(out))
    return out


def optimal_split_threshold(X, rows, j):
    """Algorithm 3: (threshold fp32, loss) for bucket `rows` of X split along column j."""
    X = _rows(X); rows = _rows_i64(rows)
    v = C.c_float(0.0); loss = C.c_double(0.0)
    _L().oracle_optimal_split_threshold(_p(X), C.c_int64(X.strides[0] // 4), C.c_int32(X.shape[1]), _p(rows),
                                        C.c_int64(rows.size), C.c_int32(j), C.byref(v), C.byref(loss))
    return np.float32(v.value), float(loss.value)


def select_idxs(X, buckets):
    """heuristic_select_idxs: candidate columns for a level whose buckets are the given row lists."""
    X = _rows(X)
    rows = _rows_i64(np.concatenate([np.asarray(b, dtype=np.int64) for b in buckets]) if buckets else [])
    start = np.zeros(len(buckets) + 1, dtype=np.int64)
    start[1:] = np.cumsum([len(b) for b in buckets])
    cand = np.zeros(4, dtype=np.int32)
    n = _L().oracle_select_idxs(_p(X), C.c_int64(X.strides[0] // 4), C.c_int32(X.shape[1]), _p(rows), _p(start),
                                C.c_int32(len(buckets)), _p(cand))
    return cand[:n].copy()


def learn_tree(X):
    """Algorithm 2 four times on the subspace matrix X: (split columns [4], thresholds [16],
    leaf - 1 of every row, l^min of every level)."""
    X = _rows(X)
    N, d = X.shape
    cols = np.zeros(4, dtype=np.int32); thr = np.zeros(16, dtype=np.float32)
    leaf = np.zeros(N, dtype=np.uint8); loss = np.zeros(4, dtype=np.float64)
    _L().oracle_learn_tree(_p(X), C.c_int64(N), C.c_int64(X.strides[0] // 4), C.c_int32(d), _p(cols), _p(thr),
                           _p(leaf), _p(loss))
    return cols, thr, leaf, loss


def _bounds(subspaces):
    b = np.ascontiguousarray(subspaces, dtype=np.int32)
    assert b.ndim == 2 and b.shape[1] == 2
    return b


def learn_trees(A, subspaces):
    """All trees: (split_dims [C][4] absolute, thresholds [C][16], codes [N][C], level losses [C][4])."""
    A = _rows(A); b = _bounds(subspaces)
    N = A.shape[0]; Cc = b.shape[0]
    sd = np.zeros((Cc, 4), dtype=np.int32); th = np.zeros((Cc, 16), dtype=np.float32)
    codes = np.zeros((N, Cc), dtype=np.uint8); loss = np.zeros((Cc, 4), dtype=np.float64)
    _L().oracle_learn_trees(_p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), C.c_int32(Cc), _p(b), _p(sd), _p(th),
                            _p(codes), _p(loss))
    return sd, th, codes, loss


def one_hot(codes, n_protos: int = 16):
    """G of Section 4.3 (fp64, N x (C n_protos)) from 0-based codes [N][C]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, Cc = codes.shape
    G = np.empty((N, Cc * n_protos), dtype=np.float64)
    _L().oracle_one_hot(_p(codes), C.c_int64(N), C.c_int32(Cc), C.c_int32(n_protos), _p(G))
    return G


def bucket_means(codes, A, subspaces):
    """Prototypes as bucket means on the codebook's own columns: fp64 [C][16][D]."""
    A = _rows(A); b = _bounds(subspaces)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, D = A.shape; Cc = b.shape[0]
    P = np.empty((Cc, 16, D), dtype=np.float64)
    _L().oracle_bucket_means(_p(codes), _p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), C.c_int32(D),
                             C.c_int32(Cc), _p(b), _p(P))
    return P


def ridge_prototypes(codes, A, lam: float = 1.0):
    """P = (G^T G + lam I)^-1 G^T A (Section 4.3): fp64 [C][16][D]."""
    A = _rows(A)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, D = A.shape; Cc = codes.shape[1]
    P = np.empty((Cc, 16, D), dtype=np.float64)
    rc = _L().oracle_ridge_prototypes(_p(codes), _p(A), C.c_int64(N), C.c_int64(A.strides[0] // 4), C.c_int32(D),
                                      C.c_int32(Cc), C.c_double(lam), _p(P))
    if rc != 0:
        raise ValueError("G^T G + lambda I is not positive definite")
    return P
