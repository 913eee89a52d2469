"""Checks of the offline learner (CPU set-up): Algorithms 2-4 and the ridge step."""
import numpy as np

import oracle
import workloads as wl
from paper_2106_10860_amd import learn as L


def two_pass_sse(X):
    X = X.astype(np.float64)
    return float(((X - X.mean(axis=0)) ** 2).sum()) if len(X) else 0.0


def test_cumulative_sse_matches_two_pass_definition():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((23, 5)).astype(np.float32)
    head = L.cumulative_sse(X, False)
    tail = L.cumulative_sse(X, True)
    for n in range(1, 24):
        assert abs(head[n - 1] - two_pass_sse(X[:n])) < 1e-9
        assert abs(tail[n - 1] - two_pass_sse(X[n - 1:])) < 1e-9


def test_optimal_split_threshold_brute_force():
    rng = np.random.default_rng(1)
    for trial in range(30):
        n = int(rng.integers(2, 32))
        X = rng.integers(0, 6, size=(n, 3)).astype(np.float32)   # many ties
        if trial % 3 == 0:
            X = rng.standard_normal((n, 3)).astype(np.float32)
        jj = int(rng.integers(0, 3))
        v, loss = L.optimal_split_threshold(X, jj)
        # brute force: every threshold between two distinct sorted values
        vals = np.unique(X[:, jj])
        best = two_pass_sse(X) if len(vals) == 1 else np.inf
        for a, b in zip(vals[:-1], vals[1:]):
            t = (a + b) / 2
            best = min(best, two_pass_sse(X[X[:, jj] < t]) + two_pass_sse(X[X[:, jj] >= t]))
        assert abs(loss - best) < 1e-6 * max(1.0, best)
        # the realised split (the >= test of Algorithm 1) has exactly that loss
        realised = two_pass_sse(X[X[:, jj] < v]) + two_pass_sse(X[X[:, jj] >= v])
        assert abs(realised - best) < 1e-6 * max(1.0, best)


def test_ridge_closed_form_single_codebook_and_normal_equations():
    rng = np.random.default_rng(2)
    A = rng.standard_normal((200, 6)).astype(np.float32)
    codes = rng.integers(0, 16, size=(200, 1))
    codes[codes == 5] = 4                                   # leave bucket 5 empty
    P = L.ridge_prototypes(L.one_hot(codes), A, lam=1.0)
    for k in range(16):
        rows = codes[:, 0] == k
        expect = A[rows].astype(np.float64).sum(axis=0) / (rows.sum() + 1.0)
        np.testing.assert_allclose(P[k], expect, rtol=1e-10, atol=1e-12)
    assert (P[5] == 0).all()
    codes3 = rng.integers(0, 16, size=(200, 3))
    G = L.one_hot(codes3)
    P3 = L.ridge_prototypes(G, A, lam=1.0)
    resid = (G.T @ G + np.eye(48)) @ P3 - G.T @ A.astype(np.float64)
    assert np.abs(resid).max() < 1e-9
    # Lemma F.3: largest singular value of the ridge solution
    smax = np.linalg.svd(P3, compute_uv=False)[0]
    assert smax <= np.linalg.svd(A.astype(np.float64), compute_uv=False)[0] / 2.0 + 1e-9


def test_learner_is_deterministic_and_consistent_with_the_oracle_encoder():
    At, A, B = wl.random_problem(5, N=300, D=24, M=4, N_train=700)
    subs = [(0, 8), (8, 16), (16, 24)]
    m1 = L.learn(At, subs)
    m2 = L.learn(At, subs)
    assert (m1.split_dims == m2.split_dims).all() and (m1.thresholds == m2.thresholds).all()
    assert (m1.prototypes == m2.prototypes).all()
    for c, (lo, hi) in enumerate(subs):
        assert ((m1.split_dims[c] >= lo) & (m1.split_dims[c] < hi)).all()
    # the buckets the learner formed are the leaves Algorithm 1 assigns
    assert (oracle.encode(At, m1.split_dims, m1.thresholds) == m1.train_codes).all()
    # every level lowers (never raises) the training SSE; ridge does not do worse
    # than the bucket means on the training rows
    pq = L.learn(At, subs, ridge=False)
    G = L.one_hot(m1.train_codes)
    err_ridge = ((G @ m1.prototypes.reshape(48, -1).astype(np.float64) - At) ** 2).sum()
    err_pq = ((G @ pq.prototypes.reshape(48, -1).astype(np.float64) - At) ** 2).sum()
    assert err_ridge <= err_pq * (1 + 1e-3) + 48 * 1.0   # ridge penalty lam * |P|^2 aside
    assert err_pq < ((At - At.mean(axis=0)) ** 2).sum()


def test_narrow_and_tiny_subspaces():
    rng = np.random.default_rng(3)
    At = rng.integers(0, 4, size=(50, 5)).astype(np.float32)
    m = L.learn(At, [(0, 2), (2, 3), (3, 5)])
    assert m.split_dims.shape == (3, 4) and (m.split_dims[1] == 2).all()
    assert np.isfinite(m.thresholds).all() and np.isfinite(m.prototypes).all()
    assert (oracle.encode(At, m.split_dims, m.thresholds) == m.train_codes).all()


def test_numpy_learner_agrees_with_the_oracle_learner():
    """The product's CPU learner (vectorised NumPy) against the oracle's plain statement of
    Algorithms 2-4 and of the ridge step, on two of the seeded workloads: split columns,
    thresholds and training codes equal, prototypes equal to fp32 rounding."""
    for cfg in (1, 6):
        w = wl.get_workload(cfg)
        At = wl.make_A_train(w)
        m = L.learn(At, w.subspaces)
        sd, th, codes, _ = oracle.learn_trees(At, w.subspaces)
        assert (sd == m.split_dims).all() and (th == m.thresholds).all() and (codes == m.train_codes).all()
        P = oracle.ridge_prototypes(codes, At, 1.0)
        np.testing.assert_allclose(m.prototypes, P, rtol=1e-6, atol=1e-7 * np.abs(P).max())
        pq = L.learn(At, w.subspaces, ridge=False)
        np.testing.assert_allclose(pq.prototypes, oracle.bucket_means(codes, At, w.subspaces), rtol=1e-6, atol=1e-9)
