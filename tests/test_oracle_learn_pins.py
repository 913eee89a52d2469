"""Pins of the oracle's LEARNING step (oracle/maddness_learn_oracle.c) to things other than
itself: the loss equation of Section 4.2, Algorithms 2-4 (Section 4.2, Appendix C) and the
ridge step of Section 4.3.  All on the CPU; the checkers are library routines, closed forms
and brute force written out here in NumPy / Python."""
import numpy as np
import pytest

import oracle


def two_pass_sse(X):
    """L(B): sum over columns and rows of (x - column mean)^2 (loss equation of Section 4.2)."""
    X = np.asarray(X, dtype=np.float64)
    return float(((X - X.mean(axis=0)) ** 2).sum()) if len(X) else 0.0


# ---------------------------------------------------------------------------
# L(j, B)
# ---------------------------------------------------------------------------

def test_bucket_loss_is_count_times_variance():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((40, 6)).astype(np.float32)
    rows = np.sort(rng.choice(40, size=17, replace=False))
    for j in range(6):
        want = 17 * np.var(X[rows, j].astype(np.float64))          # library variance
        assert abs(oracle.bucket_loss(X, rows, j) - want) < 1e-12 * max(1.0, want)
    # hand example: {1, 2, 6} has mean 3 and squared deviations 4 + 1 + 9
    H = np.array([[1.0, 5.0], [2.0, 5.0], [6.0, 5.0]], dtype=np.float32)
    assert oracle.bucket_loss(H, [0, 1, 2], 0) == 14.0
    assert oracle.bucket_loss(H, [0, 1, 2], 1) == 0.0               # a constant column
    assert oracle.bucket_loss(H, [], 0) == 0.0 and oracle.bucket_loss(H, [1], 0) == 0.0
    # only the rows of the bucket count, and a padded row stride is honoured
    wide = np.zeros((3, 5), dtype=np.float32)
    wide[:, :2] = H
    assert oracle.bucket_loss(wide[:, :2], [0, 2], 0) == 12.5


# ---------------------------------------------------------------------------
# Algorithm 4
# ---------------------------------------------------------------------------

def test_cumulative_sse_against_two_pass_sums_of_every_prefix_and_suffix():
    rng = np.random.default_rng(1)
    for n, d in ((1, 3), (2, 1), (23, 5), (64, 16)):
        X = rng.standard_normal((n, d)).astype(np.float32)
        head = oracle.cumulative_sse(X, False)
        tail = oracle.cumulative_sse(X, True)
        for i in range(n):
            assert abs(head[i] - two_pass_sse(X[:i + 1])) < 1e-9     # rows 1..n of the paper
            assert abs(tail[i] - two_pass_sse(X[i:])) < 1e-9        # rows n..N (turned back)
        assert head[0] == 0.0 and tail[-1] == 0.0                    # out_1 = 0
    # integer data: sums are exact, so the identity sum x^2 - (sum x)^2 / n holds to the last bit
    X = rng.integers(0, 256, size=(50, 4)).astype(np.float32)
    head = oracle.cumulative_sse(X, False)
    for i in range(1, 50):
        x = X[:i + 1].astype(np.float64)
        want = sum(float((x[:, c] ** 2).sum()) - float(x[:, c].sum()) ** 2 / (i + 1) for c in range(4))
        assert abs(head[i] - want) <= 1e-9 * want


def test_cumulative_sse_needs_every_column_and_the_row_itself():
    # a dropped column, or X_{1,d} instead of X_{n,d} in the inner loop, would fail here
    X = np.array([[0.0, 0.0], [0.0, 10.0], [3.0, 10.0]], dtype=np.float32)
    head = oracle.cumulative_sse(X, False)
    assert head[1] == 50.0                 # column 1: {0, 10}
    assert abs(head[2] - (6.0 + 200.0 / 3.0)) < 1e-12
    tail = oracle.cumulative_sse(X, True)
    assert tail[1] == 4.5 and tail[2] == 0.0


# ---------------------------------------------------------------------------
# Algorithm 3
# ---------------------------------------------------------------------------

def brute_force_split(X, j):
    """Minimal loss over every threshold that separates two different values of column j."""
    vals = np.unique(X[:, j])
    if len(vals) < 2:
        return two_pass_sse(X), None
    best, where = np.inf, None
    for a, b in zip(vals[:-1], vals[1:]):
        loss = two_pass_sse(X[X[:, j] <= a]) + two_pass_sse(X[X[:, j] >= b])
        if loss < best:
            best, where = loss, (a, b)
    return best, where


def test_optimal_split_threshold_brute_force():
    rng = np.random.default_rng(2)
    for trial in range(60):
        n = int(rng.integers(1, 40))
        d = int(rng.integers(1, 5))
        X = rng.integers(0, 6, size=(n, d)).astype(np.float32)          # many ties
        if trial % 3 == 0:
            X = rng.standard_normal((n, d)).astype(np.float32)
        if trial % 7 == 0:
            X = np.maximum(X - 2, 0).astype(np.float32)                  # exact zeros, as after a ReLU
        j = int(rng.integers(0, d))
        rows = np.arange(n)
        v, loss = oracle.optimal_split_threshold(X, rows, j)
        best, where = brute_force_split(X, j)
        assert abs(loss - best) <= 1e-9 * max(1.0, best), (trial, loss, best)
        if where is None:
            assert v == X[0, j]                                         # cannot be split: its value
        else:
            # the split Algorithm 1 makes with this threshold (x_j >= v goes right) has that loss
            realised = two_pass_sse(X[X[:, j] < v]) + two_pass_sse(X[X[:, j] >= v])
            assert abs(realised - best) <= 1e-9 * max(1.0, best)
            assert (X[:, j] < v).any() and (X[:, j] >= v).any()
    # a sub-bucket of a larger matrix with a padded row stride
    big = rng.standard_normal((30, 7)).astype(np.float32)
    rows = np.array([1, 4, 5, 9, 17, 18, 29])
    v, loss = oracle.optimal_split_threshold(big[:, :4], rows, 2)
    best, _ = brute_force_split(big[rows, :4], 2)
    assert abs(loss - best) < 1e-9
    assert oracle.optimal_split_threshold(big[:, :4], [], 0) == (np.float32(0.0), 0.0)


def test_threshold_is_an_fp32_number_strictly_above_the_lower_neighbour():
    # two adjacent fp32 values: their midpoint rounds to one of them; lower < v <= upper must hold
    lo = np.float32(1.0)
    hi = np.nextafter(lo, np.float32(2.0))
    X = np.array([[lo], [lo], [hi], [hi]], dtype=np.float32)
    v, loss = oracle.optimal_split_threshold(X, np.arange(4), 0)
    assert v == hi and loss == 0.0
    # first minimum wins: {0, 1, 2, 3} splits equally well after 0|123 ... no; 01|23 is the unique best
    X = np.array([[0.0], [1.0], [2.0], [3.0]], dtype=np.float32)
    v, loss = oracle.optimal_split_threshold(X, np.arange(4), 0)
    assert v == np.float32(1.5) and loss == 1.0
    # equal losses (0|12 and 01|2 for {0, 1, 2}): the first position
    X = np.array([[0.0], [1.0], [2.0]], dtype=np.float32)
    v, loss = oracle.optimal_split_threshold(X, np.arange(3), 0)
    assert v == np.float32(0.5) and loss == 0.5


# ---------------------------------------------------------------------------
# heuristic_select_idxs and Algorithm 2
# ---------------------------------------------------------------------------

def test_select_idxs_ranks_columns_by_loss_summed_over_buckets():
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((60, 7)) * np.array([1, 5, 2, 9, 0.1, 3, 4])).astype(np.float32)
    buckets = [np.arange(0, 25), np.arange(25, 60)]
    total = [sum(len(b) * np.var(X[b, j].astype(np.float64)) for b in buckets) for j in range(7)]
    want = np.argsort(-np.array(total), kind="stable")[:4]
    assert (oracle.select_idxs(X, buckets) == want).all()
    # fewer than four columns: all of them; equal losses: index order
    assert oracle.select_idxs(X[:, :2], buckets).tolist() == [1, 0]
    Z = np.zeros((10, 6), dtype=np.float32)
    assert oracle.select_idxs(Z, [np.arange(10)]).tolist() == [0, 1, 2, 3]


def python_tree(X):
    """Algorithm 2, level by level, in Python with brute-force split search: the best of the
    heuristic's candidate columns, thresholds per bucket, below / above children."""
    N, d = X.shape
    node = np.zeros(N, dtype=int)
    cols, losses = [], []
    for t in range(4):
        buckets = [np.nonzero(node == i)[0] for i in range(1 << t)]
        total = [sum(two_pass_sse(X[b][:, [j]]) for b in buckets) for j in range(d)]
        cand = np.argsort(-np.array(total), kind="stable")[:min(4, d)]
        best = (np.inf, None)
        for j in cand:
            l = sum(brute_force_split(X[b], j)[0] for b in buckets)
            if l < best[0] - 1e-9 * max(1.0, l):
                best = (l, int(j))
        cols.append(best[1]); losses.append(best[0])
        j = best[1]
        for i, b in enumerate(buckets):
            _, where = brute_force_split(X[b], j)
            above = np.zeros(len(b), dtype=bool) if where is None and len(b) == 0 else (
                np.ones(len(b), dtype=bool) if where is None else X[b, j] >= where[1])
            node[b] = 2 * i + above
    return cols, losses, node


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_tree_against_brute_force_level_by_level(seed):
    rng = np.random.default_rng(seed)
    N, d = int(rng.integers(40, 120)), int(rng.integers(2, 7))
    X = (rng.standard_normal((N, d)) * rng.uniform(0.5, 3.0, size=d)).astype(np.float32)
    if seed % 2:
        X = np.maximum(X, 0).astype(np.float32)
    cols, thr, leaf, loss = oracle.learn_tree(X)
    want_cols, want_loss, want_node = python_tree(X)
    assert cols.tolist() == want_cols
    np.testing.assert_allclose(loss, want_loss, rtol=1e-9)
    assert (leaf == want_node).all()
    assert (np.diff(loss) <= 1e-9).all()                    # a level never raises the loss
    assert loss[-1] <= two_pass_sse(X) + 1e-9
    # the buckets the learner formed are the leaves Algorithm 1 assigns with these parameters
    codes = oracle.encode(X, cols[None, :], thr[None, :])
    assert (codes[:, 0] == leaf).all()
    assert thr[15] == 0.0


def test_tree_recovers_sixteen_clusters():
    # 16 well-separated clusters along one coordinate, little spread elsewhere: the four levels
    # must cut that coordinate into the 16 clusters, in order
    rng = np.random.default_rng(5)
    centre = np.arange(16) * 10.0
    which = np.repeat(np.arange(16), 12)
    rng.shuffle(which)
    X = np.zeros((which.size, 3), dtype=np.float32)
    X[:, 1] = centre[which] + rng.uniform(-1, 1, which.size)
    X[:, 0] = rng.uniform(-0.1, 0.1, which.size)
    X[:, 2] = rng.uniform(-0.1, 0.1, which.size)
    cols, thr, leaf, loss = oracle.learn_tree(X)
    assert cols.tolist() == [1, 1, 1, 1]
    assert (leaf == which).all()
    assert abs(loss[3] - sum(two_pass_sse(X[which == k]) for k in range(16))) < 1e-9
    assert abs(thr[0] - 75.0) < 2.0                         # the root cuts between clusters 7 and 8


def test_learn_trees_over_subspaces_and_degenerate_inputs():
    rng = np.random.default_rng(6)
    A = rng.integers(0, 4, size=(50, 5)).astype(np.float32)
    subs = [(0, 2), (2, 3), (3, 5)]
    sd, th, codes, loss = oracle.learn_trees(A, subs)
    for c, (lo, hi) in enumerate(subs):
        assert ((sd[c] >= lo) & (sd[c] < hi)).all()
        cols, thr, leaf, l = oracle.learn_tree(A[:, lo:hi])
        assert (sd[c] == lo + cols).all() and (th[c] == thr).all() and (codes[:, c] == leaf).all()
    assert np.isfinite(th).all()
    assert (oracle.encode(A, sd, th) == codes).all()
    # a constant matrix: nothing can be split, every row ends in the right-most leaf (x >= v everywhere)
    Z = np.full((9, 2), 3.0, dtype=np.float32)
    sd, th, codes, loss = oracle.learn_trees(Z, [(0, 2)])
    assert (codes == 15).all() and (loss == 0).all() and (oracle.encode(Z, sd, th) == codes).all()
    # a single row
    sd, th, codes, loss = oracle.learn_trees(Z[:1], [(0, 2)])
    assert (oracle.encode(Z[:1], sd, th) == codes).all()


# ---------------------------------------------------------------------------
# prototypes: bucket means and the ridge step (Section 4.3)
# ---------------------------------------------------------------------------

def test_bucket_means():
    rng = np.random.default_rng(7)
    A = rng.standard_normal((120, 6)).astype(np.float32)
    codes = rng.integers(0, 16, size=(120, 2)).astype(np.uint8)
    codes[codes[:, 1] == 3, 1] = 4                         # bucket 3 of codebook 1 stays empty
    subs = [(0, 4), (4, 6)]
    P = oracle.bucket_means(codes, A, subs)
    for c, (lo, hi) in enumerate(subs):
        for k in range(16):
            rows = codes[:, c] == k
            want = np.zeros(6)
            if rows.any():
                want[lo:hi] = A[rows, lo:hi].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(P[c, k], want, rtol=1e-13, atol=1e-15)
    assert (P[1, 3] == 0).all()


def test_ridge_closed_form_normal_equations_and_library_solver():
    rng = np.random.default_rng(8)
    A = rng.standard_normal((200, 6)).astype(np.float32)
    codes = rng.integers(0, 16, size=(200, 1)).astype(np.uint8)
    codes[codes == 5] = 4                                   # leave bucket 5 empty
    P = oracle.ridge_prototypes(codes, A, 1.0)[0]
    # one codebook: G^T G is diagonal, so P_k = sum of the bucket's rows / (count + lambda)
    for k in range(16):
        rows = codes[:, 0] == k
        expect = A[rows].astype(np.float64).sum(axis=0) / (rows.sum() + 1.0)
        np.testing.assert_allclose(P[k], expect, rtol=1e-12, atol=1e-14)
    assert (P[5] == 0).all()
    # several codebooks: the normal equations hold, and a library solver agrees
    codes3 = rng.integers(0, 16, size=(200, 3)).astype(np.uint8)
    G = np.eye(16)[codes3].reshape(200, 48)
    for lam in (1.0, 0.25):
        P3 = oracle.ridge_prototypes(codes3, A, lam).reshape(48, 6)
        resid = (G.T @ G + lam * np.eye(48)) @ P3 - G.T @ A.astype(np.float64)
        assert np.abs(resid).max() < 1e-9
        np.testing.assert_allclose(P3, np.linalg.solve(G.T @ G + lam * np.eye(48), G.T @ A.astype(np.float64)),
                                   rtol=1e-9, atol=1e-11)
    # Lemma F.3: the largest singular value of the ridge solution is at most that of A / (2 sqrt(lambda))
    P3 = oracle.ridge_prototypes(codes3, A, 1.0).reshape(48, 6)
    assert np.linalg.svd(P3, compute_uv=False)[0] <= np.linalg.svd(A.astype(np.float64), compute_uv=False)[0] / 2 + 1e-9
    # without the penalty an empty bucket makes the system singular: reported, not returned
    with pytest.raises(ValueError):
        oracle.ridge_prototypes(codes, A, 0.0)


def test_ridge_does_not_fit_the_training_rows_worse_than_bucket_means():
    rng = np.random.default_rng(9)
    W = rng.standard_normal((4, 12))
    A = np.maximum(rng.standard_normal((600, 4)) @ W + 0.1 * rng.standard_normal((600, 12)), 0).astype(np.float32)
    subs = [(0, 4), (4, 8), (8, 12)]
    sd, th, codes, _ = oracle.learn_trees(A, subs)
    G = np.eye(16)[codes].reshape(600, 48)
    err = lambda P: float(((G @ P.reshape(48, 12) - A) ** 2).sum())
    ridge, means = oracle.ridge_prototypes(codes, A, 1.0), oracle.bucket_means(codes, A, subs)
    # ridge minimises |A - G P|^2 + lambda |P|^2 over ALL P, the bucket means are one such P
    assert err(ridge) + (ridge ** 2).sum() <= err(means) + (means ** 2).sum() + 1e-9
    assert err(means) < two_pass_sse(A)
