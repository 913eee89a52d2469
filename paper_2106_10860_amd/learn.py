"""Offline learning for MADDNESS (CPU, NumPy, untimed set-up).

Runs once per problem and produces the parameters that the inference library
consumes: split indices and thresholds of the C hashing trees (Section 4.2,
Algorithm 2; Appendix C, Algorithms 3-4) and the prototype matrix (bucket means,
Section 4; optionally refined by ridge regression, Section 4.3).  Nothing here
is on the timed path and nothing here touches the GPU.

Readings of the paper where it is silent or garbled:
  * candidate split indices come from the codebook's own subspace; the top
    n = min(4, |J|) by bucket SSE summed over buckets, ties to the lower index;
  * the loss of a split is the SSE over all dimensions of the subspace, summed
    over the two children (Algorithm 4 sums over columns);
  * split positions are only taken between two different values of the split
    column (ties all fall on one side of a >= test), the threshold is the fp32
    midpoint v with lo < v <= hi; a bucket that cannot be split keeps loss
    SSE(bucket) and gets its (single) value as threshold; an empty bucket gets 0;
  * Algorithm 4's inner loop reads row n (the printed X_{1,d} is a typo) and the
    reversed pass is flipped back so that tail[n] is the SSE of rows n..N;
  * ridge: P = (G^T G + lambda I)^-1 G^T A_train literally, lambda = 1, fp64,
    cast to fp32.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np

K = 16
DEPTH = 4
N_CANDIDATES = 4


@dataclass
class MaddnessModel:
    split_dims: np.ndarray   # int32 [C][4], absolute column of A per tree level
    thresholds: np.ndarray   # fp32  [C][16], level t (1..4) node i (1..2^(t-1)) at slot 2^(t-1)-1+(i-1)
    prototypes: np.ndarray   # fp32  [C][16][D]
    train_codes: np.ndarray  # uint8 [N_train][C], leaf - 1 of every training row

    @property
    def C(self) -> int:
        return int(self.split_dims.shape[0])

    @property
    def D(self) -> int:
        return int(self.prototypes.shape[2])


def bucket_sse_per_dim(X: np.ndarray) -> np.ndarray:
    """L(j, B) of Section 4.2 for every column j of the bucket X (two-pass form)."""
    if X.shape[0] == 0:
        return np.zeros(X.shape[1])
    Xd = X.astype(np.float64)
    return ((Xd - Xd.mean(axis=0)) ** 2).sum(axis=0)


def cumulative_sse(X: np.ndarray, reverse: bool) -> np.ndarray:
    """Algorithm 4: out[n-1] = SSE, summed over columns, of the first n rows of X
    (reverse=False) or of rows n..N (reverse=True, result flipped back)."""
    Xd = X.astype(np.float64)
    if reverse:
        Xd = Xd[::-1]
    n = np.arange(1, Xd.shape[0] + 1, dtype=np.float64)[:, None]
    cum = np.cumsum(Xd, axis=0)
    cum2 = np.cumsum(Xd * Xd, axis=0)
    out = (cum2 - cum * cum / n).sum(axis=1)
    out = np.maximum(out, 0.0)
    return out[::-1] if reverse else out


def _fp32_midpoint(lo: np.float32, hi: np.float32) -> np.float32:
    v = np.float32((np.float64(lo) + np.float64(hi)) * 0.5)
    if not (v > lo):
        v = np.float32(hi)
    return v


def optimal_split_threshold(X: np.ndarray, jj: int) -> Tuple[np.float32, float]:
    """Algorithm 3 on bucket X (rows x subspace columns), splitting column jj.

    Returns (threshold, loss)."""
    n = X.shape[0]
    if n == 0:
        return np.float32(0.0), 0.0
    order = np.argsort(X[:, jj], kind="stable")
    Xs = X[order]
    col = Xs[:, jj]
    if n < 2 or not (col[0] < col[-1]):
        return np.float32(col[0]), float(bucket_sse_per_dim(X).sum())
    head = cumulative_sse(Xs, False)      # head[i] = SSE(rows 0..i)
    tail = cumulative_sse(Xs, True)       # tail[i] = SSE(rows i..n-1)
    losses = head[:-1] + tail[1:]         # split after sorted row i, i = 0..n-2
    valid = col[:-1] < col[1:]
    losses = np.where(valid, losses, np.inf)
    i = int(np.argmin(losses))
    return _fp32_midpoint(col[i], col[i + 1]), float(losses[i])


def _learn_tree(X: np.ndarray):
    """Greedy construction of one tree on the subspace matrix X (N x |J|).

    Returns (local split columns [4], thresholds fp32 [16] in heap order, leaf of
    every row in 0..15)."""
    N, d = X.shape
    split_cols = np.zeros(DEPTH, dtype=np.int64)
    thr = np.zeros(16, dtype=np.float32)
    node = np.zeros(N, dtype=np.int64)           # 0-based node index within the level
    for t in range(DEPTH):
        n_nodes = 1 << t
        members = [np.nonzero(node == i)[0] for i in range(n_nodes)]
        # heuristic_select_idxs: columns with the most SSE summed over buckets
        per_dim = np.zeros(d)
        for rows in members:
            per_dim += bucket_sse_per_dim(X[rows])
        n_cand = min(N_CANDIDATES, d)
        cand = np.argsort(-per_dim, kind="stable")[:n_cand]
        best_loss, best_j, best_v = np.inf, int(cand[0]), None
        for jj in cand:
            vs = np.zeros(n_nodes, dtype=np.float32)
            loss = 0.0
            for i, rows in enumerate(members):
                vs[i], li = optimal_split_threshold(X[rows], int(jj))
                loss += li
            if loss < best_loss or best_v is None:
                best_loss, best_j, best_v = loss, int(jj), vs
        split_cols[t] = best_j
        thr[n_nodes - 1: 2 * n_nodes - 1] = best_v
        above = X[:, best_j] >= best_v[node]
        node = 2 * node + above.astype(np.int64)
    return split_cols, thr, node


def one_hot(codes: np.ndarray, n_protos: int = K) -> np.ndarray:
    """Matrix G of Section 4.3: row n is the concatenation of the one-hot
    encodings of codes[n][c] (0-based) over the codebooks."""
    N, C = codes.shape
    G = np.zeros((N, C * n_protos), dtype=np.float64)
    G[np.arange(N)[:, None], np.arange(C)[None, :] * n_protos + codes] = 1.0
    return G


def ridge_prototypes(G: np.ndarray, A_train: np.ndarray, lam: float = 1.0) -> np.ndarray:
    """P = (G^T G + lam I)^-1 G^T A_train  (Section 4.3), fp64."""
    from scipy.linalg import cho_factor, cho_solve

    GtG = G.T @ G
    GtG[np.diag_indices_from(GtG)] += lam
    rhs = G.T @ A_train.astype(np.float64)
    return cho_solve(cho_factor(GtG, lower=True), rhs)


def learn(A_train: np.ndarray, subspaces: Sequence[Tuple[int, int]], ridge: bool = True,
          lam: float = 1.0) -> MaddnessModel:
    """Learn trees and prototypes from the training matrix.

    subspaces: [start, stop) column range of every codebook (disjoint).
    ridge=False keeps the block-diagonal bucket means (the ablation the paper
    calls MADDNESS-PQ, Section 5.1)."""
    A_train = np.ascontiguousarray(A_train, dtype=np.float32)
    N, D = A_train.shape
    C = len(subspaces)
    split_dims = np.zeros((C, 4), dtype=np.int32)
    thresholds = np.zeros((C, 16), dtype=np.float32)
    codes = np.zeros((N, C), dtype=np.uint8)
    for c, (lo, hi) in enumerate(subspaces):
        cols, thr, leaf = _learn_tree(A_train[:, lo:hi])
        split_dims[c] = lo + cols
        thresholds[c] = thr
        codes[:, c] = leaf
    P = np.zeros((C, K, D), dtype=np.float64)
    if ridge:
        P = ridge_prototypes(one_hot(codes), A_train, lam).reshape(C, K, D)
    else:
        for c, (lo, hi) in enumerate(subspaces):
            for k in range(K):
                rows = codes[:, c] == k
                if rows.any():
                    P[c, k, lo:hi] = A_train[rows, lo:hi].astype(np.float64).mean(axis=0)
    return MaddnessModel(split_dims, thresholds, np.ascontiguousarray(P, dtype=np.float32), codes)
