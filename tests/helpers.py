"""Shared plumbing of the GPU parity tests: run the same bytes through the CPU
oracle and through the C ABI of the HIP library, and compare."""
from __future__ import annotations

import numpy as np

import oracle

REL_TOL = 1e-6   # fp32 outputs: relative error bound of the build's target


def random_trees(rng, A_like: np.ndarray, C: int):
    """Random split dims and thresholds drawn from the data's own values (so that
    ties between data and thresholds occur, as they do for learned trees)."""
    N, D = A_like.shape
    sd = rng.integers(0, D, size=(C, 4)).astype(np.int32)
    th = np.zeros((C, 16), dtype=np.float32)
    for c in range(C):
        for t in range(4):
            vals = A_like[rng.integers(0, N, size=1 << t), sd[c, t]]
            th[c, (1 << t) - 1:(1 << (t + 1)) - 1] = vals
    return sd, th


def oracle_pipeline(A, sd, th, P, B):
    """Everything the path computes, on the CPU.  Returns a dict of host arrays."""
    C = sd.shape[0]
    codes = oracle.encode(A, sd, th)
    packed = oracle.pack(codes)
    T = oracle.build_luts_f64(P, B)
    luts, scale, offset, l, delta = oracle.quantize_luts(T)
    out, acc, ov = oracle.scan(packed, C, luts, scale, offset)
    assert ov == 0
    return dict(codes=codes, packed=packed, T=T, luts=luts, scale=scale, offset=offset, l=l,
                delta=delta, out=out, acc=acc)


def assert_out_close(got: np.ndarray, want: np.ndarray, what: str):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    tol = REL_TOL * np.abs(want.astype(np.float64))
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outputs beyond {REL_TOL} relative; " \
                          f"worst {err.max():.3e}"


def compare_luts(got_luts, got_scale, got_offset, ref, P, B):
    """Parity rule for the table build: the GPU contracts in fp64 on the matrix
    cores, the oracle in fp64 sequentially, so T differs by summation order only.
    scale must be equal; offset equal to fp32 rounding of a sum that differs by
    <= 1e-12 relative; a byte may differ by 1 only where the oracle's value before
    rounding is within 1e-9 of a half-integer.  Returns the number of such bytes."""
    assert (got_scale == ref["scale"]).all(), "scale differs"
    np.testing.assert_allclose(got_offset, ref["offset"], rtol=2e-7, atol=1e-30)
    diff = got_luts.astype(np.int32) - ref["luts"].astype(np.int32)
    if not diff.any():
        return 0
    assert np.abs(diff).max() <= 1, "table entry differs by more than one level"
    pre = (ref["T"] - ref["delta"][:, None, :]) * (2.0 ** ref["l"].astype(np.float64))[None, None, :]
    frac = np.abs(pre - np.floor(pre) - 0.5)
    assert (frac[diff != 0] < 1e-9).all(), "table entry differs away from a rounding boundary"
    return int((diff != 0).sum())
