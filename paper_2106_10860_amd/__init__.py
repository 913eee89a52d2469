"""Python binding of libmaddness (the C ABI in ``include/maddness.h``).

Argument marshalling only: every function below checks tensor types, takes the
raw device pointers and calls the entry point of the same name; all of the
method's arithmetic runs in the HIP kernels.  PyTorch is used for device memory
and streams, nothing else.  There is no CPU fallback: if the shared library is
missing or a call fails, an exception is raised.

The offline learner (CPU, untimed set-up) is in ``paper_2106_10860_amd.learn``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaddness.so")

MADDNESS_OK = 0
MADDNESS_E_INVAL = -1
MADDNESS_E_UNSUPPORTED = -2
MADDNESS_E_ALIGN = -3
MADDNESS_E_HIP = -4

EXPORTS = (
    "maddness_encode",
    "maddness_build_luts_workspace",
    "maddness_build_luts",
    "maddness_build_luts_pooled",
    "maddness_build_luts_static",
    "maddness_scan",
    "maddness_encode_scan",
    "maddness_scan_averaged",
    "maddness_encode_scan_averaged",
    "maddness_encode_typed",
    "maddness_encode_scan_typed",
    "maddness_learn_trees_workspace",
    "maddness_learn_trees",
    "maddness_learn_prototypes_workspace",
    "maddness_learn_prototypes",
    "maddness_set_option",
    "maddness_get_option",
    "maddness_last_error",
    "maddness_last_kernel",
)


class MaddnessError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"maddness status {status}: {text}")
        self.status = status


class _Params(C.Structure):
    _fields_ = [("D", C.c_int32), ("C", C.c_int32), ("split_dims", C.c_void_p),
                ("thresholds", C.c_void_p), ("prototypes", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Loads libmaddness.so (built in-tree by ``build.py``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2106_10860_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.maddness_encode.argtypes = [C.POINTER(_Params), vp, i64, i64, vp, vp]
        L.maddness_build_luts_workspace.argtypes = [i32, i32, i32]
        L.maddness_build_luts_workspace.restype = sz
        L.maddness_build_luts.argtypes = [C.POINTER(_Params), vp, i32, i64, vp, vp, vp, vp, sz, vp]
        L.maddness_build_luts_pooled.argtypes = L.maddness_build_luts.argtypes
        L.maddness_build_luts_static.argtypes = [C.POINTER(_Params), vp, i32, i64, vp, vp, vp, vp]
        L.maddness_scan.argtypes = [i32, i32, vp, i64, vp, vp, vp, vp, i64, vp, vp]
        L.maddness_encode_scan.argtypes = [C.POINTER(_Params), vp, i64, i64, i32, vp, vp, vp, vp, i64,
                                           vp, vp, vp]
        L.maddness_scan_averaged.argtypes = L.maddness_scan.argtypes
        L.maddness_encode_scan_averaged.argtypes = L.maddness_encode_scan.argtypes
        L.maddness_encode_typed.argtypes = [C.POINTER(_Params), vp, i32, i32, i64, i64, vp, vp]
        L.maddness_encode_scan_typed.argtypes = [C.POINTER(_Params), vp, i32, i32, i64, i64, i32, vp, vp, vp,
                                                 vp, i64, vp, vp, vp]
        L.maddness_learn_trees_workspace.argtypes = [i64, i32, i32, vp]
        L.maddness_learn_trees_workspace.restype = sz
        L.maddness_learn_trees.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.maddness_learn_prototypes_workspace.argtypes = [i32, i32]
        L.maddness_learn_prototypes_workspace.restype = sz
        L.maddness_learn_prototypes.argtypes = [vp, vp, i64, i64, i32, i32, vp, i32, C.c_double, vp, vp, sz, vp]
        L.maddness_set_option.argtypes = [i32, i32]
        L.maddness_get_option.argtypes = [i32]
        L.maddness_get_option.restype = i32
        L.maddness_last_error.restype = C.c_char_p
        L.maddness_last_kernel.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != MADDNESS_OK:
        raise MaddnessError(status, lib().maddness_last_error().decode())


def _ptr(t, dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if dtype == torch.uint16 and t.dtype == torch.int16:
        return t.data_ptr()      # same bytes; int16 tensors have wider operator support
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, has {t.dtype}")
    return t.data_ptr()


def _rows(t, name: str):
    """(pointer, row stride in elements) of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with unit column stride")
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0)))


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


class Params:
    """Learned parameters resident on the device (see ``maddness_params``)."""

    def __init__(self, split_dims, thresholds, prototypes=None):
        import torch
        self.C = int(split_dims.shape[0])
        if tuple(split_dims.shape) != (self.C, 4) or tuple(thresholds.shape) != (self.C, 16):
            raise ValueError("split_dims must be [C][4] and thresholds [C][16]")
        self.split_dims = split_dims.contiguous()
        self.thresholds = thresholds.contiguous()
        self.prototypes = None if prototypes is None else prototypes.contiguous()
        if prototypes is not None:
            if prototypes.dim() != 3 or prototypes.shape[0] != self.C or prototypes.shape[1] != 16:
                raise ValueError("prototypes must be [C][16][D]")
        self.D: Optional[int] = None if prototypes is None else int(prototypes.shape[2])
        self._c = None
        self._torch = torch

    @classmethod
    def from_model(cls, model, device="cuda"):
        """Uploads a ``learn.MaddnessModel`` (host NumPy arrays)."""
        import torch
        return cls(torch.from_numpy(model.split_dims).to(device),
                   torch.from_numpy(model.thresholds).to(device),
                   torch.from_numpy(model.prototypes).to(device))

    def c_struct(self, D: int) -> _Params:
        t = self._torch
        return _Params(D, self.C, _ptr(self.split_dims, t.int32, "split_dims"),
                       _ptr(self.thresholds, t.float32, "thresholds"),
                       _ptr(self.prototypes, t.float32, "prototypes"))


def maddness_encode(params: Params, A, codes=None, stream=None):
    """g(A): packed 4-bit codes, uint8 [N][(C+1)/2]."""
    import torch
    N, D, lda = _rows(A, "A")
    if params.D is not None and params.D != D:
        raise ValueError("A has a different D than the prototypes")
    if codes is None:
        codes = torch.empty((N, (params.C + 1) // 2), dtype=torch.uint8, device=A.device)
    p = params.c_struct(D)
    _check(lib().maddness_encode(C.byref(p), _ptr(A, torch.float32, "A"), N, lda,
                                 _ptr(codes, torch.uint8, "codes"), _stream(stream)))
    return codes


MADDNESS_F32, MADDNESS_F16, MADDNESS_BF16, MADDNESS_U8 = 0, 1, 2, 3
MADDNESS_ROW_MAJOR, MADDNESS_COL_MAJOR = 0, 1


def _typed(A, col_major: bool):
    """(pointer, dtype code, layout code, N, D, lda) of an input of any supported type.
    With col_major the tensor holds the columns of A: shape [D][N]."""
    import torch
    codes = {torch.float32: MADDNESS_F32, torch.float16: MADDNESS_F16, torch.bfloat16: MADDNESS_BF16,
             torch.uint8: MADDNESS_U8}
    if not isinstance(A, torch.Tensor) or not A.is_cuda:
        raise TypeError("A must be a device tensor")
    if A.dtype not in codes:
        raise TypeError(f"A has dtype {A.dtype}; supported: float32, float16, bfloat16, uint8")
    r, c, ld = _rows(A, "A")
    N, D = (c, r) if col_major else (r, c)
    return A.data_ptr(), codes[A.dtype], (MADDNESS_COL_MAJOR if col_major else MADDNESS_ROW_MAJOR), N, D, ld


def maddness_encode_typed(params: Params, A, col_major=False, codes=None, stream=None):
    """g(A) for A of dtype float32 / float16 / bfloat16 / uint8, stored by rows ([N][D]) or,
    with col_major, by columns ([D][N])."""
    import torch
    ptr, dt, layout, N, D, lda = _typed(A, col_major)
    if params.D is not None and params.D != D:
        raise ValueError("A has a different D than the prototypes")
    if codes is None:
        codes = torch.empty((N, (params.C + 1) // 2), dtype=torch.uint8, device=A.device)
    p = params.c_struct(D)
    _check(lib().maddness_encode_typed(C.byref(p), ptr, dt, layout, N, lda, _ptr(codes, torch.uint8, "codes"),
                                       _stream(stream)))
    return codes


def maddness_encode_scan_typed(params: Params, A, luts, scale, offset, col_major=False, out=None, acc=None,
                               codes=None, want_out=True, stream=None):
    """Fused g, f and alpha f + beta for A of any supported type and storage order."""
    import torch
    ptr, dt, layout, N, D, lda = _typed(A, col_major)
    M = luts.shape[2]
    if want_out and out is None:
        out = torch.empty((N, M), dtype=torch.float32, device=A.device)
    ldo = 0 if out is None else _rows(out, "out")[2]
    p = params.c_struct(D)
    _check(lib().maddness_encode_scan_typed(C.byref(p), ptr, dt, layout, N, lda, M,
                                            _ptr(luts, torch.uint8, "luts"),
                                            _ptr(scale, torch.float32, "scale"),
                                            _ptr(offset, torch.float32, "offset"),
                                            _ptr(out, torch.float32, "out"), ldo,
                                            _ptr(acc, torch.uint16, "acc"),
                                            _ptr(codes, torch.uint8, "codes"), _stream(stream)))
    return out


def maddness_build_luts_pooled(params: Params, B, luts=None, scale=None, offset=None, workspace=None,
                               stream=None):
    """h(B) quantised as Appendix A prints it: one scale, one offset per codebook."""
    return maddness_build_luts(params, B, luts, scale, offset, workspace, stream, _pooled=True)


def maddness_build_luts(params: Params, B, luts=None, scale=None, offset=None, workspace=None,
                        stream=None, _pooled=False):
    """h(B): uint8 tables [C][16][M] with per-column scale and offset."""
    import torch
    D, M, ldb = _rows(B, "B")
    if params.D != D:
        raise ValueError("B has a different D than the prototypes")
    dev = B.device
    luts = torch.empty((params.C, 16, M), dtype=torch.uint8, device=dev) if luts is None else luts
    scale = torch.empty(M, dtype=torch.float32, device=dev) if scale is None else scale
    offset = torch.empty(M, dtype=torch.float32, device=dev) if offset is None else offset
    need = lib().maddness_build_luts_workspace(D, params.C, M)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    p = params.c_struct(D)
    entry = lib().maddness_build_luts_pooled if _pooled else lib().maddness_build_luts
    _check(entry(C.byref(p), _ptr(B, torch.float32, "B"), M, ldb,
                 _ptr(luts, torch.uint8, "luts"), _ptr(scale, torch.float32, "scale"),
                 _ptr(offset, torch.float32, "offset"), _ptr(workspace, torch.uint8, "workspace"),
                 workspace.numel(), _stream(stream)))
    return luts, scale, offset


STATIC_WORKSPACE_BYTES = 8388608


def maddness_build_luts_static(params: Params, B, luts, scale, offset, stream=None):
    """h(B) with the library's own per-GPU workspace: the call allocates nothing, so every
    output is passed in.  Shapes beyond STATIC_WORKSPACE_BYTES raise MADDNESS_E_UNSUPPORTED."""
    import torch
    D, M, ldb = _rows(B, "B")
    if params.D != D:
        raise ValueError("B has a different D than the prototypes")
    if tuple(luts.shape) != (params.C, 16, M) or scale.numel() != M or offset.numel() != M:
        raise ValueError("luts must be [C][16][M], scale and offset [M]")
    p = params.c_struct(D)
    _check(lib().maddness_build_luts_static(C.byref(p), _ptr(B, torch.float32, "B"), M, ldb,
                                            _ptr(luts, torch.uint8, "luts"), _ptr(scale, torch.float32, "scale"),
                                            _ptr(offset, torch.float32, "offset"), _stream(stream)))
    return luts, scale, offset


def _scan(entry, n_codebooks: int, codes, luts, scale, offset, out, acc, want_out, stream):
    import torch
    N = codes.shape[0]
    M = luts.shape[2]
    if want_out and out is None:
        out = torch.empty((N, M), dtype=torch.float32, device=codes.device)
    ldo = 0 if out is None else _rows(out, "out")[2]
    _check(entry(n_codebooks, M, _ptr(codes, torch.uint8, "codes"), N,
                 _ptr(luts, torch.uint8, "luts"), _ptr(scale, torch.float32, "scale"),
                 _ptr(offset, torch.float32, "offset"),
                 _ptr(out, torch.float32, "out"), ldo,
                 _ptr(acc, torch.uint16, "acc"), _stream(stream)))
    return out, acc


def maddness_scan(n_codebooks: int, codes, luts, scale, offset, out=None, acc=None, want_out=True,
                  stream=None):
    """f and alpha f + beta from packed codes.  Returns (out, acc); either may be None."""
    return _scan(lib().maddness_scan, n_codebooks, codes, luts, scale, offset, out, acc, want_out, stream)


def maddness_scan_averaged(n_codebooks: int, codes, luts, scale, offset, out=None, acc=None,
                           want_out=True, stream=None):
    """As maddness_scan with the pairwise-average aggregation (blocks of 16 codebooks)."""
    return _scan(lib().maddness_scan_averaged, n_codebooks, codes, luts, scale, offset, out, acc,
                 want_out, stream)


def _encode_scan(entry, params: Params, A, luts, scale, offset, out, acc, codes, want_out, stream):
    import torch
    N, D, lda = _rows(A, "A")
    M = luts.shape[2]
    if want_out and out is None:
        out = torch.empty((N, M), dtype=torch.float32, device=A.device)
    ldo = 0 if out is None else _rows(out, "out")[2]
    p = params.c_struct(D)
    _check(entry(C.byref(p), _ptr(A, torch.float32, "A"), N, lda, M,
                 _ptr(luts, torch.uint8, "luts"),
                 _ptr(scale, torch.float32, "scale"),
                 _ptr(offset, torch.float32, "offset"),
                 _ptr(out, torch.float32, "out"), ldo,
                 _ptr(acc, torch.uint16, "acc"),
                 _ptr(codes, torch.uint8, "codes"), _stream(stream)))
    return out


def maddness_encode_scan(params: Params, A, luts, scale, offset, out=None, acc=None, codes=None,
                         want_out=True, stream=None):
    """Fused g, f and alpha f + beta.  Returns out (or None when want_out is False)."""
    return _encode_scan(lib().maddness_encode_scan, params, A, luts, scale, offset, out, acc, codes,
                        want_out, stream)


def maddness_encode_scan_averaged(params: Params, A, luts, scale, offset, out=None, acc=None, codes=None,
                                  want_out=True, stream=None):
    """As maddness_encode_scan with the pairwise-average aggregation (blocks of 16 codebooks)."""
    return _encode_scan(lib().maddness_encode_scan_averaged, params, A, luts, scale, offset, out, acc,
                        codes, want_out, stream)


def _bounds(subspaces):
    """HOST int32 array [C][2] of (first, one-past-last) columns."""
    flat = [int(v) for pair in subspaces for v in pair]
    if len(flat) % 2 or not flat:
        raise ValueError("subspaces must be a non-empty sequence of (first, one-past-last) pairs")
    return (C.c_int32 * len(flat))(*flat), len(flat) // 2


def maddness_learn_trees(A_train, subspaces, split_dims=None, thresholds=None, train_codes=None, workspace=None,
                         stream=None):
    """The C hashing trees from a training matrix on the device (Section 4.2; Appendix C).
    Returns device tensors (split_dims int32 [C][4], thresholds fp32 [C][16], train_codes uint8 [N][C])."""
    import torch
    N, D, lda = _rows(A_train, "A_train")
    bounds, n_cb = _bounds(subspaces)
    dev = A_train.device
    split_dims = torch.empty((n_cb, 4), dtype=torch.int32, device=dev) if split_dims is None else split_dims
    thresholds = torch.empty((n_cb, 16), dtype=torch.float32, device=dev) if thresholds is None else thresholds
    train_codes = torch.empty((N, n_cb), dtype=torch.uint8, device=dev) if train_codes is None else train_codes
    need = lib().maddness_learn_trees_workspace(N, D, n_cb, bounds)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib().maddness_learn_trees(_ptr(A_train, torch.float32, "A_train"), N, lda, D, n_cb, bounds,
                                      _ptr(split_dims, torch.int32, "split_dims"),
                                      _ptr(thresholds, torch.float32, "thresholds"),
                                      _ptr(train_codes, torch.uint8, "train_codes"),
                                      _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))
    return split_dims, thresholds, train_codes


def maddness_learn_prototypes(train_codes, A_train, subspaces, ridge=True, lam=1.0, prototypes=None, workspace=None,
                              stream=None):
    """The prototypes [C][16][D] from the training codes: ridge regression (Section 4.3) or, with
    ridge=False, the bucket means."""
    import torch
    N, D, lda = _rows(A_train, "A_train")
    bounds, n_cb = _bounds(subspaces)
    if tuple(train_codes.shape) != (N, n_cb):
        raise ValueError("train_codes must be [N][C], one byte per code")
    dev = A_train.device
    prototypes = torch.empty((n_cb, 16, D), dtype=torch.float32, device=dev) if prototypes is None else prototypes
    need = lib().maddness_learn_prototypes_workspace(D, n_cb)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib().maddness_learn_prototypes(_ptr(train_codes.contiguous(), torch.uint8, "train_codes"),
                                           _ptr(A_train, torch.float32, "A_train"), N, lda, D, n_cb, bounds,
                                           1 if ridge else 0, float(lam), _ptr(prototypes, torch.float32, "prototypes"),
                                           _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                           _stream(stream)))
    return prototypes


def learn_on_device(A_train, subspaces, ridge=True, lam=1.0, stream=None) -> "Params":
    """Both learning calls on a training matrix that is resident on the device; returns the
    parameters as the inference calls take them (still on the device)."""
    split_dims, thresholds, codes = maddness_learn_trees(A_train, subspaces, stream=stream)
    prototypes = maddness_learn_prototypes(codes, A_train, subspaces, ridge=ridge, lam=lam, stream=stream)
    return Params(split_dims, thresholds, prototypes)


MADDNESS_OPT_KERNELS, MADDNESS_OPT_PHASED_ROWS, MADDNESS_OPT_COLS_RUN, MADDNESS_OPT_MAX_WORKGROUPS = 0, 1, 2, 3
MADDNESS_KERNELS_AUTO, MADDNESS_KERNELS_NO_MATRIX_CORES, MADDNESS_KERNELS_GENERAL = 0, 1, 2


def maddness_set_option(option: int, value: int) -> None:
    """Process-wide kernel-selection switch for tests and measurements (never changes a result)."""
    _check(lib().maddness_set_option(option, value))


def maddness_get_option(option: int) -> int:
    return lib().maddness_get_option(option)


def maddness_last_kernel() -> str:
    """Which kernel the last call on this thread launched (diagnostic; "" if none)."""
    return lib().maddness_last_kernel().decode()
