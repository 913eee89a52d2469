"""Seeded generators for the five synthetic workloads (see package docstring).

All randomness comes from ``numpy.random.Generator(Philox(seed))`` with the
seeds listed in ``WORKLOADS``; a chunk of A can be regenerated on its own, so
the large workloads never need the whole matrix on the host at once.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

CHUNK = 65536


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # "latent_relu", "image" or "series"
    N: int               # rows of A
    D: int               # columns of A / rows of B
    M: int               # columns of B
    C: int               # codebooks
    N_train: int         # rows of the training matrix
    latent: int          # latent dimension (latent_relu only)
    seed_W: int
    seed_train: int
    seed_A: int          # seed of chunk 0; chunk i uses seed_A + i
    seed_B: int
    chunked: bool        # True: A is drawn in CHUNK-row pieces
    subspaces: Tuple[Tuple[int, int], ...] = field(default=())  # [start, stop) per codebook


def _even_subspaces(D: int, C: int) -> Tuple[Tuple[int, int], ...]:
    w = D // C
    assert w * C == D
    return tuple((c * w, (c + 1) * w) for c in range(C))


WORKLOADS = {
    1: Workload("cfg1_softmax10", "latent_relu", 10000, 512, 10, 16, 5000, 64,
                1000, 1001, 1002, 1003, False, _even_subspaces(512, 16)),
    2: Workload("cfg2_softmax100", "latent_relu", 10000, 512, 100, 32, 5000, 64,
                2000, 2001, 2002, 2003, False, _even_subspaces(512, 32)),
    3: Workload("cfg3_image3x3", "image", 510 * 510, 27, 2, 4, 510 * 510, 0,
                0, 3001, 3002, 0, False, ((0, 7), (7, 14), (14, 21), (21, 27))),
    4: Workload("cfg4_throughput", "latent_relu", 1 << 20, 512, 256, 32, 20000, 64,
                4000, 4001, 4100, 4003, True, _even_subspaces(512, 32)),
    5: Workload("cfg5_stress", "latent_relu", 1 << 22, 1024, 512, 64, 32768, 128,
                5000, 5001, 5100, 5003, True, _even_subspaces(1024, 64)),
    # shape of the paper's time-series task (Appendix E.5): series resampled to length
    # 320, 1000 test rows, B = 128 exemplar series
    6: Workload("cfg6_series_kernel", "series", 1000, 320, 128, 16, 2000, 0,
                6000, 6001, 6002, 6003, False, _even_subspaces(320, 16)),
}


def get_workload(i: int) -> Workload:
    return WORKLOADS[i]


def n_chunks(w: Workload) -> int:
    return (w.N + CHUNK - 1) // CHUNK if w.chunked else 1


def chunk_rows(w: Workload, i: int) -> Tuple[int, int]:
    """Row range [lo, hi) of chunk ``i``."""
    if not w.chunked:
        assert i == 0
        return 0, w.N
    lo = i * CHUNK
    return lo, min(w.N, lo + CHUNK)


# ----------------------------------------------------------------------------
# latent-ReLU rows: A = max(0, Z W + 0.1 E)
# ----------------------------------------------------------------------------

def _latent_W(w: Workload) -> np.ndarray:
    g = _rng(w.seed_W)
    return (g.standard_normal((w.latent, w.D), dtype=np.float32)
            / np.float32(np.sqrt(w.latent))).astype(np.float32)


def _latent_rows(w: Workload, n: int, seed: int, W: np.ndarray) -> np.ndarray:
    g = _rng(seed)
    Z = g.standard_normal((n, w.latent), dtype=np.float32)
    A = Z @ W
    # noise drawn in pieces so that the temporary stays small
    step = 16384
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        E = g.standard_normal((hi - lo, w.D), dtype=np.float32)
        A[lo:hi] += np.float32(0.1) * E
    np.maximum(A, np.float32(0.0), out=A)
    return np.ascontiguousarray(A, dtype=np.float32)


# ----------------------------------------------------------------------------
# image rows: every valid 3x3 window of a smooth 512x512 RGB image, CHW order
# ----------------------------------------------------------------------------

def _smooth_image(seed: int, side: int = 512) -> np.ndarray:
    from scipy.ndimage import gaussian_filter

    g = _rng(seed)
    img = g.random((side, side, 3))
    out = np.empty((3, side, side), dtype=np.float32)
    for ch in range(3):
        b = gaussian_filter(img[:, :, ch], sigma=3.0, mode="reflect")
        b = (b - b.min()) / (b.max() - b.min()) * 255.0
        out[ch] = np.rint(b).astype(np.uint8).astype(np.float32)
    return out  # CHW, integer values 0..255 held in fp32


def _windows_chw(img: np.ndarray, k: int = 3) -> np.ndarray:
    ch, H, W = img.shape
    v = np.lib.stride_tricks.sliding_window_view(img, (k, k), axis=(1, 2))  # ch, H-k+1, W-k+1, k, k
    v = v.transpose(1, 2, 0, 3, 4)  # y, x, ch, ky, kx
    return np.ascontiguousarray(v.reshape((H - k + 1) * (W - k + 1), ch * k * k), dtype=np.float32)


def _image_B() -> np.ndarray:
    sobel_x = np.array([[-1, 0, 1], [-2, 0, 2], [-1, 0, 1]], dtype=np.float64)
    ax = np.arange(-1, 2, dtype=np.float64)
    g1 = np.exp(-0.5 * ax * ax)
    gauss = np.outer(g1, g1)
    gauss /= gauss.sum()
    B = np.empty((27, 2), dtype=np.float32)
    B[:, 0] = np.tile(sobel_x.reshape(-1), 3)
    B[:, 1] = np.tile(gauss.reshape(-1), 3)
    return B


# ----------------------------------------------------------------------------
# series rows: z-normalised smooth time series from a handful of classes
# ----------------------------------------------------------------------------

def _series_rows(w: Workload, n: int, seed: int) -> np.ndarray:
    """n series of length D: one of 8 class shapes (4 sinusoids each, fixed by seed_W),
    shifted in time by a random amount, plus smoothed noise; every row has mean 0 and
    standard deviation 1, as the series of the archive the paper uses do."""
    from scipy.ndimage import gaussian_filter1d

    gs = _rng(w.seed_W)
    n_classes = 8
    freq = gs.uniform(0.5, 6.0, size=(n_classes, 4))
    amp = gs.uniform(0.3, 1.0, size=(n_classes, 4))
    phase = gs.uniform(0.0, 2 * np.pi, size=(n_classes, 4))
    g = _rng(seed)
    cls = g.integers(0, n_classes, size=n)
    shift = g.uniform(-0.05, 0.05, size=n)
    t = np.arange(w.D, dtype=np.float64) / w.D
    tt = t[None, :] + shift[:, None]
    X = np.zeros((n, w.D), dtype=np.float64)
    for h in range(4):
        X += amp[cls, h][:, None] * np.sin(2 * np.pi * freq[cls, h][:, None] * tt + phase[cls, h][:, None])
    X += 0.3 * gaussian_filter1d(g.standard_normal((n, w.D)), sigma=2.0, axis=1, mode="reflect")
    X -= X.mean(axis=1, keepdims=True)
    X /= X.std(axis=1, keepdims=True)
    return np.ascontiguousarray(X, dtype=np.float32)


# ----------------------------------------------------------------------------
# public entry points
# ----------------------------------------------------------------------------

def make_B(w: Workload) -> np.ndarray:
    if w.kind == "image":
        return _image_B()
    if w.kind == "series":
        # columns = exemplar series (the paper learns them from the training set; here
        # they are further draws of the same generator)
        return np.ascontiguousarray(_series_rows(w, w.M, w.seed_B).T)
    g = _rng(w.seed_B)
    return (g.standard_normal((w.D, w.M), dtype=np.float32)
            / np.float32(np.sqrt(w.D))).astype(np.float32)


def make_A_train(w: Workload) -> np.ndarray:
    if w.kind == "image":
        return _windows_chw(_smooth_image(w.seed_train))
    if w.kind == "series":
        return _series_rows(w, w.N_train, w.seed_train)
    return _latent_rows(w, w.N_train, w.seed_train, _latent_W(w))


def make_A_chunk(w: Workload, i: int) -> np.ndarray:
    lo, hi = chunk_rows(w, i)
    if w.kind == "image":
        return _windows_chw(_smooth_image(w.seed_A))
    if w.kind == "series":
        return _series_rows(w, w.N, w.seed_A)
    return _latent_rows(w, hi - lo, w.seed_A + i, _latent_W(w))


def make_A(w: Workload) -> np.ndarray:
    if not w.chunked:
        return make_A_chunk(w, 0)
    out = np.empty((w.N, w.D), dtype=np.float32)
    for i in range(n_chunks(w)):
        lo, hi = chunk_rows(w, i)
        out[lo:hi] = make_A_chunk(w, i)
    return out


def random_problem(seed: int, N: int, D: int, M: int, latent: int = 8, N_train: int = 512):
    """Small latent-ReLU problem of arbitrary shape for edge-case tests.

    Returns (A_train, A, B), all fp32, C-contiguous.
    """
    g = _rng(seed)
    W = (g.standard_normal((latent, D), dtype=np.float32) / np.float32(np.sqrt(latent)))

    def rows(n):
        Z = g.standard_normal((n, latent), dtype=np.float32)
        E = g.standard_normal((n, D), dtype=np.float32)
        return np.ascontiguousarray(np.maximum(Z @ W + np.float32(0.1) * E, 0), dtype=np.float32)

    A_train = rows(N_train)
    A = rows(N)
    B = (g.standard_normal((D, M), dtype=np.float32) / np.float32(np.sqrt(D))).astype(np.float32)
    return A_train, A, np.ascontiguousarray(B)
