"""Properties that the definitions force on the CPU oracle, checked on drawn inputs.

Each is an identity of the mathematics (exact in the arithmetic used), not a comparison of the oracle
with itself on the same input: a changed input must change the output in the stated way.
"""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

SETTINGS = dict(max_examples=25, deadline=None)


def _trees(rng, D, C):
    sd = rng.integers(0, D, size=(C, 4)).astype(np.int32)
    th = np.zeros((C, 16), np.float32)
    th[:, :15] = rng.integers(-8, 9, size=(C, 15)).astype(np.float32)
    return sd, th


@settings(**SETTINGS)
@given(st.integers(0, 2**31 - 1), st.integers(1, 5), st.integers(-64, 64), st.integers(-3, 3))
def test_codes_survive_an_increasing_map_of_data_and_thresholds(seed, C, shift, log2_factor):
    """Algorithm 1 only compares: x -> 2^s x + k (exact on small integers), applied to the data and to
    the thresholds alike, changes no comparison (Section 4.1)."""
    rng = np.random.default_rng(seed)
    N, D = 50, 7
    A = rng.integers(-10, 11, size=(N, D)).astype(np.float32)
    sd, th = _trees(rng, D, C)
    f = np.float32(2.0 ** log2_factor)
    A2 = A * f + np.float32(shift)
    th2 = th.copy()
    th2[:, :15] = th[:, :15] * f + np.float32(shift)
    assert (oracle.encode(A, sd, th) == oracle.encode(A2, sd, th2)).all()


@settings(**SETTINGS)
@given(st.integers(0, 2**31 - 1), st.integers(2, 9), st.integers(1, 6))
def test_scan_is_additive_over_a_split_of_the_codebooks(seed, C, M):
    """f sums one entry per codebook (Section 4.4): the sums over two groups of codebooks add up."""
    rng = np.random.default_rng(seed)
    N = 40
    codes = rng.integers(0, 16, size=(N, C)).astype(np.uint8)
    luts = rng.integers(0, 256, size=(C, 16, M)).astype(np.uint8)
    scale = np.ones(M, np.float32)
    offset = np.zeros(M, np.float32)
    k = int(rng.integers(1, C))
    _, acc, ov = oracle.scan(oracle.pack(codes), C, luts, scale, offset)
    _, acc1, _ = oracle.scan(oracle.pack(codes[:, :k]), k, np.ascontiguousarray(luts[:k]), scale, offset)
    _, acc2, _ = oracle.scan(oracle.pack(codes[:, k:]), C - k, np.ascontiguousarray(luts[k:]), scale, offset)
    assert ov == 0
    assert (acc.astype(np.int64) == acc1.astype(np.int64) + acc2.astype(np.int64)).all()


@settings(**SETTINGS)
@given(st.integers(0, 2**31 - 1), st.integers(-20, 20))
def test_quantisation_follows_a_power_of_two_rescaling(seed, s):
    """Appendix A: the scale is the power of two that fits the widest table, so T -> 2^s T keeps every
    byte, and multiplies scale and offset by 2^s (all exact)."""
    rng = np.random.default_rng(seed)
    C, M = 3, 4
    T = rng.standard_normal((C, 16, M))
    luts, scale, offset, l, delta = oracle.quantize_luts(T)
    luts2, scale2, offset2, l2, delta2 = oracle.quantize_luts(np.ldexp(T, s))
    assert (luts == luts2).all()
    assert (l2 == l - s).all()
    assert (scale2 == np.ldexp(scale, s)).all()
    assert (delta2 == np.ldexp(delta, s)).all()
    assert (offset2 == np.ldexp(offset, s).astype(np.float32)).all()


@settings(**SETTINGS)
@given(st.integers(0, 2**31 - 1), st.integers(-50, 50))
def test_quantisation_moves_a_table_shift_into_the_offset(seed, k):
    """Appendix A subtracts each table's minimum: adding a constant to the 16 entries of one (codebook,
    column) table changes no byte and adds the constant to that column's offset (dyadic values: exact)."""
    rng = np.random.default_rng(seed)
    C, M = 4, 3
    T = rng.integers(-64, 65, size=(C, 16, M)).astype(np.float64) / 8.0
    c, m = int(rng.integers(C)), int(rng.integers(M))
    T2 = T.copy()
    T2[c, :, m] += k / 4.0
    luts, scale, offset, _, delta = oracle.quantize_luts(T)
    luts2, scale2, offset2, _, delta2 = oracle.quantize_luts(T2)
    assert (luts == luts2).all() and (scale == scale2).all()
    want = delta.copy()
    want[c, m] += k / 4.0
    assert (delta2 == want).all()
    assert offset2[m] == np.float32(delta2[:, m].sum()) and (np.delete(offset2, m) == np.delete(offset, m)).all()


@settings(**SETTINGS)
@given(st.integers(0, 2**31 - 1))
def test_rows_are_independent(seed):
    """Every step of the path treats rows independently (Appendix E.2): a row's outputs do not depend on
    which other rows are present, nor on its position."""
    rng = np.random.default_rng(seed)
    N, D, C, M = 30, 6, 3, 4
    A = rng.integers(-5, 6, size=(N, D)).astype(np.float32)
    sd, th = _trees(rng, D, C)
    luts = rng.integers(0, 256, size=(C, 16, M)).astype(np.uint8)
    scale = np.ldexp(np.ones(M, np.float32), -3)
    offset = rng.standard_normal(M).astype(np.float32)
    out, acc, packed = oracle.encode_scan(A, sd, th, luts, scale, offset)
    pick = rng.permutation(N)[: N // 2]
    out2, acc2, packed2 = oracle.encode_scan(np.ascontiguousarray(A[pick]), sd, th, luts, scale, offset)
    assert (out2 == out[pick]).all() and (acc2 == acc[pick]).all() and (packed2 == packed[pick]).all()
